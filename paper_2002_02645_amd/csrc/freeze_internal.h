// Internal declarations shared by the translation units of the library
// (host dispatcher <-> kernel launchers).  Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace fz {

constexpr int kTileN = 256;      // cache entries per matrix-core tile; cache rows are padded to it
constexpr int kPadD = 64;        // activation length is padded to a multiple of this (bf16 copies)
constexpr int kKB = 32;          // elements per k-block of the tiled bf16 layout (64 bytes per row piece)

// Tiled bf16 operand layout (cache and prepared queries).  A matrix of rows x d_pad is stored as
//   [row tile][k-block][row in tile][32 elements]
// so that the operands of one k-step of one tile are one contiguous run of memory that the
// distance kernel copies verbatim into LDS.  Inside each 64-byte row piece the four 16-byte
// chunks are XOR-swizzled with a function of the row so that the fragment reads of the 16x16x32
// matrix-core operands (lane l: row l & 15, chunk l >> 4) run at the full ds_read_b128 rate
// (measured: 195 B/clk/CU with this function, 128 without a swizzle).
__host__ __device__ inline int tiled_chunk_swizzle(int row)
{
    return (row >> 1) & 3;
}
// Offset, in 16-byte chunks, of logical chunk `j` (elements 8j .. 8j+7) of row `row_in_tile`
// inside a row tile of `tile_rows` rows.
__host__ __device__ inline int64_t tiled_chunk_offset(int row_in_tile, int64_t j, int tile_rows)
{
    const int64_t kb = j >> 2;
    const int c = (int)(j & 3);
    return (kb * tile_rows + row_in_tile) * 4 + (c ^ tiled_chunk_swizzle(row_in_tile));
}
// fp32 -> bf16, round to nearest even (inputs are finite by contract; NaN stays NaN)
__device__ __forceinline__ uint16_t bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
// LDS-direct 16-byte load: lane i reads 16 bytes at sbase + voff (scalar 64-bit base, 32-bit
// per-lane offset: half the address traffic of a 64-bit per-lane pointer) and they land in LDS at
// lds_byte_addr + 16 i.  M0 carries the wave-uniform LDS destination.  Issued through inline asm:
// the compiler would otherwise order every LDS read behind the outstanding direct loads; the
// kernels count their loads themselves (wait_global_loads_le).
__device__ __forceinline__ void load16_global_to_lds(uint64_t sbase, uint32_t voff, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}
// the same with the non-temporal hint (data that no other workgroup will ask for again)
__device__ __forceinline__ void load16_global_to_lds_nt(uint64_t sbase, uint32_t voff, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_byte_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}
__device__ __forceinline__ uint64_t uniform_u64(uint64_t x)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}
// Wait until at most N of this wave's global loads are outstanding (loads complete in order).
template <int N>
__device__ __forceinline__ void wait_global_loads_le() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

constexpr int kMaxRescore = 64;  // largest re-scoring width R
constexpr int kMaxK = 64;
constexpr int kMaxMergeEntries = 8192;  // n_splits * R gathered per query in the finishing kernel
constexpr int kSkinnyRows = 16;         // small-batch (bandwidth-bound) path: at most this many queries ...
constexpr int kSkinnyMaxD = 1024;       // ... and at most this padded activation length
constexpr uint64_t kSentinel = ~0ull;   // "no entry" in (key, index) lists; larger than every real entry
// Exactness certificate of the bf16 pre-filter (see finish_kernel): candidates re-scored when the
// first certificate fails, the width of the error margin in estimated standard deviations, and the
// fewest (distinct) samples an estimate is taken from.
constexpr int kTier1 = 256;
constexpr double kCertZ = 8.0;
constexpr int kCertMinSamples = 8;
constexpr int kScanMaxSplits = 512;     // exact scan of a flagged query: at most this many workgroups share it

// One layer's cache inside the caller's storage buffer.
struct LayerCache {
    bool built = false;
    int64_t n = 0, d = 0;
    int64_t n_pad = 0, d_pad = 0;
    int32_t num_classes = 0;
    int entries_dtype = 0;
    const uint16_t *c_bf = nullptr;   // n_pad x d_pad bf16, zero padded, tiled layout (tiles of kTileN rows)
    const float *norm = nullptr;      // [n_pad] sum of squares of the bf16 row, fp32
    const int32_t *labels = nullptr;  // [n]
    const float *c_f32 = nullptr;     // [n, d_pad] fp32 rows when the cache was given in fp32, else null
    const uint16_t *c_rows = nullptr; // [n, d_pad] row-major bf16 rows when the cache was given in bf16, else null
    // k-means cache: the entries are cluster centres, labels their majority labels, and
    const float *fraction = nullptr;  // [n] the share of each cluster that carries its majority label (else null)
    // projection (a dense layer in front of the look-up): the entries are the rows of W and
    const float *bias = nullptr;      // [n_pad] its bias, zero padded (else null); not a cache: look-ups reject it
    // the matrix-core copy c_bf (and norm) is taken relative to this vector, and so must the queries' bf16
    const float *mu = nullptr;        // [d_pad] copy be: the cache's mean, or all zeros (decided on the device); null: none
};

// Number of splits of the cache tiles for `live_mt` live query tiles.  Units (query tile, split)
// run one per CU in rounds of num_cus; every split restarts its top-R lists and adds entries to
// the merge, so among the candidates s_j = floor(j * num_cus / live_mt), j = 1..4 (j rounds of
// workgroups), take the first, and a later one only if it fills the CUs more than 10% better
// (measured on C2: at equal fill, 12 and 19 splits are 12-15% slower than 6).  Evaluated
// identically on the host (sizing) and on the device (cascade: the live count is only known there).
__host__ __device__ inline int splits_for(int live_mt, int n_tiles, int num_cus, int max_splits)
{
    if (live_mt < 1) return 1;
    const int cap = n_tiles < max_splits ? n_tiles : max_splits;
    int best_s = 1;
    long long best_num = 0, best_den = 1;   // fill = num / den
    for (int j = 1; j <= 4; ++j) {
        int s = (int)(((long long)j * num_cus) / live_mt);
        if (s < 1) s = 1;
        if (s > cap) s = cap;
        const long long units = (long long)live_mt * s;
        const long long rounds = (units + num_cus - 1) / num_cus;
        const long long tiles_per_unit = (n_tiles + s - 1) / s;
        const long long num = (long long)live_mt * n_tiles;
        const long long den = rounds * num_cus * tiles_per_unit;
        if (best_num == 0 || num * best_den * 10 > best_num * den * 11) {   // > 10% better fill
            best_num = num;
            best_den = den;
            best_s = s;
        }
    }
    return best_s;
}

// Which distance kernel variant serves a re-scoring width.
struct DistPlan {
    int variant;    // 0: R<=16, 1: R<=32, 2: R<=64 (fused top-R); 3: keys-out (selection by separate kernels)
    int bm;         // queries per tile
    int r;          // entries kept per (query, split)
    int m_tiles;    // ceil(b / bm)
    int n_tiles;    // ceil(n / kTileN)
    int n_splits;   // ranges of cache tiles scanned by separate workgroups (for all m_tiles live)
    int alloc_splits;   // largest n_splits over every possible live count (stride of the lists)
    int grid_units;     // largest live_mt * n_splits over every possible live count (grid size)
    int max_splits;     // cap on n_splits (merge capacity)
    int num_cus;
    int64_t b_pad;  // m_tiles * bm
    // stream-K (keys-out variant, one query tile, cache tiles that fill the CUs badly): sk_wgs
    // workgroups each take sk_len consecutive k-steps of the flattened (cache tile, k-step) space
    // and leave their accumulators in up to sk_slots slots; a second kernel adds them up per
    // tile and emits the keys.  sk_wgs == 0: off.
    int sk_wgs, sk_len, sk_slots;
    // Balanced decomposition (fused variants; only when the live count is known on the host):
    // bal_f workgroups per query tile cut cache tiles [0, bal_nfull) evenly and bal_wgs - m_tiles *
    // bal_f more cut the flattened remainder of all query tiles, so every CU gets the same number of
    // tiles (+-1); a query then has bal_lists candidate lists.  bal_f == 0: off.
    int bal_f, bal_nfull, bal_wgs, bal_lists;
};

// d_pad decides stream-K for the keys-out variant (pass 0 to leave it off).
DistPlan plan_dist(int64_t b, int64_t n, int r, int num_cus, bool keys_out, int64_t d_pad = 0);
void plan_stream_k(DistPlan &pl, int num_cus, int64_t d_pad);   // sets the sk_* fields of a keys-out plan
size_t dist_partial_bytes(const DistPlan &plan);   // stream-K accumulator slots (0 when off)

struct DistArgs {
    const uint16_t *q_bf;   // b_pad x d_pad, tiled layout (tiles of plan.bm rows)
    const uint16_t *c_bf;   // n_pad x d_pad, tiled layout (tiles of kTileN rows)
    const float *norm;      // [n_pad]
    uint64_t *part;         // [b_pad, alloc_splits, r] packed (ordered key, index) (fused variants)
    float *keys;            // [b_pad, n_pad] every key (keys-out variant)
    uint64_t *bmin;         // [b_pad, n_pad / 32] block minima (keys-out variant)
    float *partial;         // dist_partial_bytes(plan) bytes of scratch (keys-out variant under stream-K)
    bool projection;        // keys-out variant as a projection: keys = acc + norm[col] (norm holds the bias), no bmin
    bool relu;              // ... through max(., 0)
    bool balanced;          // use the plan's balanced decomposition (needs lists >= plan.bal_lists)
    int lists;              // candidate lists per query `part` has room for (their stride); fused variants
    const int32_t *count;   // device: number of live queries, or null (= b)
    int b;
    int n;
    int d_pad;
};

// mu [d_pad] float and stats [2 d_pad] double: the centring vector and its scratch, or null (no centring);
// centre_mode 1: centre when the cache's mean dominates its spread, 2: always
hipError_t launch_cache_build(const void *entries, int dtype, int64_t n, int64_t d, int64_t n_pad, int64_t d_pad,
                              uint16_t *c_bf, float *norm, float *c_f32, uint16_t *c_rows, const int32_t *labels_in,
                              int32_t *labels_out, float *mu, double *stats, int centre_mode, hipStream_t s);

// Also clears what the later kernels of the look-up count in: flag_count[0 .. 2) and tickets[0 .. b)
// (each may be null).
// mu: the cache's centring vector [d_pad] (subtracted before the rounding) or null.
hipError_t launch_query_prep(const float *queries, const int32_t *sel, const int32_t *count, int64_t b,
                             int64_t b_pad, int bm, int64_t d, int64_t d_pad, uint16_t *q_bf, int32_t *flag_count,
                             int32_t *tickets, const float *mu, hipStream_t s);

hipError_t launch_dist_topr(const DistPlan &plan, const DistArgs &a, hipStream_t s);

// Small-batch (bandwidth-bound) path: streaming kernel + threshold + filter; the result is a
// candidate list per query for the finishing kernel.
struct SkinnyLaunch {
    const float *queries;   // [b, d] fp32: converted to bf16 by every workgroup as it starts
    int64_t d;
    const uint16_t *c_bf;
    const float *norm;
    const float *mu;        // the cache's centring vector or null
    uint64_t *bmin;         // [b, n_pad / 32] out: smallest (ordered key, index) of every block of 32 entries
    uint64_t *wgmin;        // [b, n_splits] out: smallest block minimum written by each workgroup
    int32_t *flag_count;    // cleared by the kernel (with tickets[0 .. 2 * kSkinnyRows)) for the kernels after it
    int32_t *tickets;
    int b, n, d_pad, r, n_splits;
    int64_t n_pad;
};
bool skinny_supported(int64_t b, int64_t n_pad, int64_t d_pad, int r, int num_cus);
// Selection from materialised keys (keys-out variant of the tiled kernel): threshold from the
// block minima, then the candidate lists.  b queries, rows of n_pad keys.
bool select_supported(int64_t n_pad, int r);
size_t select_workspace_bytes(int64_t rows, int64_t n_pad, int r, size_t align);
hipError_t launch_select(const float *keys, const uint64_t *bmin, int64_t n_pad, int n, int b, int r,
                         int32_t *cand_count, uint64_t *cand, hipStream_t s);
int plan_skinny_splits(int64_t n, int num_cus);
size_t skinny_workspace_bytes(int64_t n_pad, int r, size_t align);
hipError_t launch_skinny_stream(const SkinnyLaunch &a, hipStream_t s);   // block minima

struct FinishArgs {
    const uint64_t *part;   // [b_pad, alloc_splits, r]; or, with part_count, [b, part_stride] candidate lists
    const int32_t *part_count;   // device: entries per query in `part` (null: n_splits * r each)
    int part_stride;
    int n_splits, r;
    int alloc_splits;            // stride (in lists) between queries in `part`
    // with a device-side live count the number of splits is re-derived from it (splits_for):
    int bm, n_tiles, num_cus, max_splits;
    const float *queries;   // [*, d] fp32 (original batch)
    const int32_t *sel;     // compact position -> row of `queries`, or null
    const int32_t *count;   // device live-query count or null
    int b;
    int n;                  // cache entries (candidate indices are checked against it)
    int64_t d, d_pad;
    const uint16_t *c_rows; // row-major bf16 rows (cache given in bf16)
    const float *c_f32;     // non-null: re-score against the fp32 rows (cache given in fp32)
    const int32_t *labels;
    int k, vote_threshold;
    int weighted;           // 0: plurality count and vote_threshold; 1: distance-weighted confidence;
                            // 2: k-means cache (k = 1): confidence = fraction[nearest centre] / distance
    const float *fraction;  // [n] (rule 2)
    float conf_threshold;   // weighted rule: hit iff confidence > conf_threshold
    float *out_conf;        // [b] (compact order), weighted rule only
    int32_t *out_labels;    // [b] (compact order)
    uint8_t *out_hit;
    int32_t *out_votes;
    int32_t *out_nbr_idx;   // [b, k]
    float *out_nbr_dist;    // [b, k]
    // Queries whose result the certificate could not confirm, by their (compact) positions: list 0
    // (flag_list, counted in flag_count[0]) is redone by the wider re-scoring, list 1 (flag_list2,
    // flag_count[1]) by the exact scan.  The first kernel of the look-up clears both counts.
    int32_t *flag_count;    // [2]
    int32_t *flag_list;     // [b]
    int32_t *flag_list2;    // [b]
    unsigned long long *stats;   // device, [3] or null: queries confirmed after the first re-scoring, after
                                 // the wider one, and queries handed to the exact scan (added to, never cleared)
};

hipError_t launch_finish(const FinishArgs &a, int num_cus, hipStream_t s);
// Exact scan of the flagged queries (a.flag_list2 / a.flag_count[1]): brute-force fp32 distances to every
// entry, the k nearest, the label and hit decision, written over the outputs of those queries.
// tickets [b] int32 (zero on entry, zero again afterwards), part_x scan_scratch_entries(b, k, num_cus) u64.
size_t scan_scratch_entries(int64_t b, int k, int num_cus);
hipError_t launch_exact_scan(const FinishArgs &a, int32_t *tickets, uint64_t *part_x, int num_cus, hipStream_t s);
// Small-batch path: from the block minima [b, nb] and the per-group minima to the outputs (takes
// a.r blocks).  cand and samp are scratch (skinny_finish_workspace_bytes covers both); tickets
// [16] int32 must be zero on entry and are left zero.
size_t skinny_finish_workspace_bytes(int r, size_t align);
hipError_t launch_skinny_finish(const FinishArgs &a, const uint64_t *bmin, const uint64_t *wgmin, int64_t nb,
                                int n_groups, int n_tiles, uint64_t *cand, uint64_t *samp, int32_t *tickets, hipStream_t s);

hipError_t launch_compact(const uint8_t *hit, const int32_t *sel_in, const int32_t *count_in, int64_t count_max,
                          int32_t *sel_out, int32_t *count_out, int64_t *hits_out, hipStream_t s);

hipError_t launch_cascade_init(int32_t *out_labels, int32_t *out_exit, int64_t b, hipStream_t s);

hipError_t launch_cascade_scatter(const int32_t *labels, const uint8_t *hit, const int32_t *sel,
                                  const int32_t *count, int64_t b, int layer_pos, int32_t *out_labels,
                                  int32_t *out_exit, hipStream_t s);

// k-means cache build (the assignment step is the look-up itself)
// sizes [k], offsets [k + 1] and members [n] int32 are scratch
hipError_t launch_kmeans_update(const float *points, const int32_t *assign, int64_t n, int64_t d, int64_t k,
                                const float *old_centers, float *new_centers, int32_t *sizes, int32_t *offsets,
                                int32_t *members, hipStream_t s);
hipError_t launch_kmeans_majority(const int32_t *assign, const int32_t *labels, int64_t n, int num_classes, int64_t k,
                                  int32_t *majority, float *fraction, int64_t *sizes, hipStream_t s);
hipError_t launch_copy_rows_f32(const float *src, int64_t src_stride, float *dst, int64_t rows, int64_t d, hipStream_t s);
hipError_t launch_fill_i32(int32_t *dst, int32_t v, int64_t n, hipStream_t s);
hipError_t launch_copy_i32(const int32_t *src, int32_t *dst, int64_t n, hipStream_t s);

hipError_t launch_gather_rows(const float *x, int64_t d, const int32_t *sel, const int32_t *count, int64_t max_count,
                              float *out, hipStream_t s);
hipError_t launch_threshold_init(float *thr, int n, hipStream_t s);
hipError_t launch_threshold_max(const int32_t *pred, const float *conf, const int32_t *model_labels, int64_t b,
                                float *thr, hipStream_t s);

}  // namespace fz
