// Distance pass for small batches (at most 16 queries): the bandwidth-bound path.
//
// With a handful of queries the look-up is a matrix-vector product: every cache entry is
// read once and used for a few dot products, so this path is built around streaming the
// cache from HBM exactly once with many bytes in flight, not around the matrix cores' rate,
// and nothing in the streaming kernel depends on the data.
//
//  1. dist_skinny_kernel streams the cache, forms per query b and entry n the ranking key
//         key(b, n) = |c_n|^2 - 2 * sum_i Q_bf[b,i] * C_bf[n,i]     (bf16 x bf16 -> fp32 MFMA)
//     and writes, per block of 32 entries, only the smallest (key, index) pair of the block
//     (8 bytes per 32 entries and query against 64 d bytes read): stores share the counter the
//     kernel waits on for its loads, so every store it does not make keeps the stream running.
//  2. The finishing kernel of this path (skinny_tail_kernel, with the other finishing code)
//     finds the R-th smallest block minimum T.  R blocks hold an entry <= T, so the R-th
//     smallest entry overall is <= T, and every entry <= T lies in one of exactly those R
//     blocks: their 32 R entries are a superset of the R best.  It re-scores all of them
//     exactly in fp32 (d <= 1024: one KiB or two per entry), keeps the k nearest, and checks
//     that no entry outside those blocks can be nearer (every one has a key >= T).
// The threshold kernel at the end of this file serves the keys-out variant of the tiled kernel
// (one query tile), where the keys are materialised: block_threshold_kernel finds, per query, the
// R-th smallest block minimum T and collects the entries with (key, index) <= T (at most 32 R,
// all of them in the R blocks whose minimum is <= T) into a candidate list, which the general
// finishing kernel sorts, cuts to R and re-scores.
//
// Paper: Sec. 3 (k nearest neighbours of the layer output), Sec. 5 "Cache lookup
// performance" (look-up latency decides whether freezing pays off).
//
// Streaming kernel: one workgroup per range of 256-entry cache tiles, two workgroups per CU.
// The prepared queries (16 rows; the matrix cores' other 16 rows are fed zeros from registers)
// stay resident in LDS.  The
// cache, stored in the tiled layout ([tile][k-block][row][32 elements]), is one contiguous
// stream per workgroup: it is copied verbatim into a ring of NS 16 KiB LDS stages with
// LDS-direct loads, NS-1 stages in flight, and the ring keeps running across tile boundaries.
// Each of the 8 waves owns 32 of the tile's 256 entries: one 32x32x16 MFMA per 16 elements of
// k.  The tile's squared norms travel the same way (one LDS-direct load per wave and tile), so
// no ordinary load ever drains the ring.
#include "freeze_internal.h"
#include "select_common.h"

namespace fz {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void *lds_void_ptr;

namespace {

__device__ __forceinline__ void load4_global_to_lds(const void *g, uint32_t lds_byte_addr)
{
    // lane i lands at +4*i
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_byte_addr), "v"(g)
                 : "memory", "m0");
}
constexpr int kQRows = kSkinnyRows;        // query rows held in LDS (the MFMA's rows 16..31 are zero registers)
constexpr int kStage = kTileN * kKB * 2;   // 16 KiB: one k-block of one cache tile
constexpr int kNormBuf = 2 * 8 * 256;      // 4 KiB: per tile parity and wave, 64 floats
static_assert(kSkinnyRows <= 16, "queries occupy the first two row groups of the MFMA output");

template <int DMAX_, int NS_>
struct SkinnyCfg {
    static constexpr int DMAX = DMAX_, NS = NS_;
    static constexpr int A_BYTES = kQRows * DMAX * 2;
    static constexpr int LDS_BYTES = A_BYTES + kNormBuf + NS * kStage;
    static_assert(LDS_BYTES <= 81920, "two workgroups per CU");
    static_assert(NS >= 2 && NS <= 8, "stages");
};

struct SkinnyArgs {
    const float *queries;   // [b, d] fp32
    int64_t d;
    const uint16_t *c_bf;
    const float *norm;
    const float *mu;        // [d_pad] the cache's mean vector when its matrix-core copy is centred (zeros when not), or null
    uint64_t *bmin;         // [b, n_pad / 32] smallest (ordered key, index) of each block of 32 entries
    uint64_t *wgmin;        // [b, n_splits] smallest of the block minima each workgroup wrote
    int32_t *flag_count;    // cleared here for the finishing kernels: the count of flagged queries ...
    int32_t *tickets;       // ... and 2 * kSkinnyRows tickets
    int b, d_pad, n_tiles, n_splits;
    int64_t n_pad;
};

template <class C>
__global__ __launch_bounds__(512) void dist_skinny_kernel(SkinnyArgs p)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::LDS_BYTES];
    __shared__ uint64_t wmin_s[8][kQRows];   // per wave and query row: smallest block minimum so far
    const bf16x8 *smem16 = reinterpret_cast<const bf16x8 *>(smem);
    constexpr int NORMS = C::A_BYTES;                                       // byte offset of the norm buffers
    const float *normbuf = reinterpret_cast<const float *>(smem + NORMS);   // [2][8 waves][64]
    constexpr int RING = NORMS + kNormBuf;                                  // byte offset of the stage ring

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sp = blockIdx.x;
    const int nt0 = (int)(((int64_t)sp * p.n_tiles) / p.n_splits);
    const int nt1 = (int)(((int64_t)(sp + 1) * p.n_tiles) / p.n_splits);
    const int kblocks = p.d_pad / kKB;                 // k-blocks per tile
    const int total = (nt1 - nt0) * kblocks;           // stages this workgroup streams
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void_ptr)smem;

    // the cache stream of this workgroup is contiguous: tiles nt0..nt1-1, each kblocks * 16 KiB
    const uint64_t stream = uniform_u64((uint64_t)(uintptr_t)p.c_bf + (size_t)nt0 * kTileN * p.d_pad * 2);
    const uint32_t lane_off = w * 1024 + lane * 16;
    auto issue = [&](int slot, int gstep) {
        // 16 KiB = 16 wave-instructions of 1 KiB: two per wave
        const uint64_t src = stream + (size_t)gstep * kStage;
        const uint32_t dst = smem_base + RING + slot * kStage + w * 1024;
        load16_global_to_lds_nt(src, lane_off, dst);   // every byte of the cache is read once
        load16_global_to_lds_nt(src + 8192, lane_off, dst + 8192);
    };
    constexpr int LPS = 2;   // loads per wave and stage
    // norms of this wave's 32 entries of tile `t` -> normbuf[t & 1][w][lane] (lanes 32..63 duplicate)
    auto issue_norms = [&](int t) {
        load4_global_to_lds(p.norm + (size_t)t * kTileN + w * 32 + (lane & 31),
                            smem_base + NORMS + ((t & 1) * 8 + w) * 256);
    };

    if (sp == 0 && tid < 2 * kSkinnyRows + 2) {
        if (tid < 2 * kSkinnyRows) p.tickets[tid] = 0;
        else p.flag_count[tid - 2 * kSkinnyRows] = 0;   // both lists' counts
    }
    // the stream starts before the queries are converted: its first stages are on their way meanwhile
    if (total > 0) issue_norms(nt0);
#pragma unroll
    for (int ps = 0; ps < C::NS - 1; ++ps)
        if (ps < total) issue(ps, ps);

    // queries -> LDS: bf16 (round to nearest even) in the tiled layout with one 16-row tile, rows
    // past the batch and elements past d zero.  Every workgroup converts them for itself (32 KiB of
    // L2-resident reads), which saves a kernel launch in front of a 0.2 ms look-up.
    {
        uint4 *dst = reinterpret_cast<uint4 *>(smem);
        const int chunks = p.d_pad / 8;   // 16-byte chunks per row
        const bool vec = (p.d % 4) == 0;
        for (int i = tid; i < kQRows * chunks; i += 512) {
            const int row = i / chunks, j = i - row * chunks;
            const int64_t i0 = (int64_t)j * 8;
            const float *src = p.queries + (int64_t)row * p.d;
            float x[8];
            if (row < p.b && vec && i0 + 8 <= p.d) {
                const float4 v0 = *reinterpret_cast<const float4 *>(src + i0);
                const float4 v1 = *reinterpret_cast<const float4 *>(src + i0 + 4);
                x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
                x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = (row < p.b && i0 + e < p.d) ? src[i0 + e] : 0.f;
            }
            if (p.mu && row < p.b) {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] -= p.mu[i0 + e];   // (zero past d)
            }
            uint4 v;
            v.x = (uint32_t)bf16_rne(x[0]) | ((uint32_t)bf16_rne(x[1]) << 16);
            v.y = (uint32_t)bf16_rne(x[2]) | ((uint32_t)bf16_rne(x[3]) << 16);
            v.z = (uint32_t)bf16_rne(x[4]) | ((uint32_t)bf16_rne(x[5]) << 16);
            v.w = (uint32_t)bf16_rne(x[6]) | ((uint32_t)bf16_rne(x[7]) << 16);
            dst[tiled_chunk_offset(row, j, kQRows)] = v;
        }
    }
    const int g = lane >> 5;
    const int rowA = lane & 15;              // lanes whose MFMA row is 16..31 supply zeros instead
    const bool has_q = (lane & 31) < kQRows;
    const int rowB = w * 32 + (lane & 31);
    const int rdA = rowA * 4, pcxA = g ^ tiled_chunk_swizzle(rowA);
    const int rdB = rowB * 4, pcxB = g ^ tiled_chunk_swizzle(rowB);

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    uint64_t run_min[8];   // per accumulator row of this half-wave: smallest block minimum so far
#pragma unroll
    for (int e = 0; e < 8; ++e) run_min[e] = kSentinel;
    int slot = 0, kb = 0, nt = nt0;
    for (int gs = 0; gs < total; ++gs) {
        // stage gs must have landed; up to NS-2 younger stages may stay in flight
        const int younger = total - 1 - gs;
        switch (younger < C::NS - 2 ? younger : C::NS - 2) {
        case 0: wait_global_loads_le<0>(); break;
        case 1: wait_global_loads_le<1 * LPS>(); break;
        case 2: wait_global_loads_le<2 * LPS>(); break;
        case 3: wait_global_loads_le<3 * LPS>(); break;
        case 4: wait_global_loads_le<4 * LPS>(); break;
        case 5: wait_global_loads_le<5 * LPS>(); break;
        default: wait_global_loads_le<6 * LPS>(); break;
        }
        __syncthreads();
        // The norms of the NEXT tile are requested at this tile's first step, before this step's
        // stage loads: they are older than every stage still in flight when they are read, and an
        // extra outstanding load only makes the counted waits above stricter.  Each wave reads and
        // refills only its own part of the buffer.
        if (kb == 0 && nt + 1 < nt1) issue_norms(nt + 1);
        if (gs + C::NS - 1 < total) issue((slot + C::NS - 1) % C::NS, gs + C::NS - 1);

        const int baseA = kb * (kQRows * 4) + rdA;
        const int baseB = (RING + slot * kStage) / 16 + rdB;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            bf16x8 af = smem16[baseA + ((kk << 1) ^ pcxA)];
            if (!has_q) af = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            const bf16x8 bfr = smem16[baseB + ((kk << 1) ^ pcxB)];
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc, 0, 0, 0);
        }
        slot = (slot + 1 == C::NS) ? 0 : slot + 1;
        if (++kb < kblocks) continue;

        // ---- tile finished: emit the minimum (key, index) of each block of 32 entries ----
        kb = 0;
        const int n0 = nt * kTileN;
        // With fewer k-blocks than stages in flight the norm load may still be outstanding.
        if (kblocks < C::NS) wait_global_loads_le<0>();
        const float nrm = normbuf[((nt & 1) * 8 + w) * 64 + (lane & 31)];
        ++nt;
#pragma unroll
        for (int e = 0; e < 8; ++e) {   // accumulator rows 0..15: the rows that can hold a query
            const int row_lo = (e >> 2) * 8 + (e & 3);   // row held by lanes 0..31; lanes 32..63 hold row_lo + 4
            if (row_lo < p.b) {                           // uniform
                const int row = row_lo + g * 4;
                const float key = __builtin_fmaf(-2.f, acc[e], nrm);
                const bool live = row < p.b;
                // block minimum over the 32 lanes of each half-wave (xor offsets < 32 stay inside it)
                const uint32_t ob = ordered_bits(key);
                uint32_t mn = ob;
#pragma unroll
                for (int off = 16; off >= 1; off >>= 1) {
                    const uint32_t o = (uint32_t)__shfl_xor((int)mn, off, 64);
                    mn = o < mn ? o : mn;
                }
                const uint64_t eq = __ballot(ob == mn);
                const uint32_t half = (uint32_t)(g ? (eq >> 32) : (eq & 0xffffffffull));
                const int first = __builtin_ctz(half);   // lowest column holding the minimum
                const uint64_t pr = ((uint64_t)mn << 32) | (uint32_t)(n0 + w * 32 + first);
                run_min[e] = pr < run_min[e] ? pr : run_min[e];
                if (live && (lane & 31) == 0) p.bmin[(size_t)row * (p.n_pad / 32) + (size_t)(n0 / 32) + w] = pr;
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    }
    // the workgroup's smallest block minimum per query (the finishing kernel starts from these)
    if ((lane & 31) == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) wmin_s[w][(e >> 2) * 8 + (e & 3) + g * 4] = run_min[e];
    }
    __syncthreads();
    if (tid < p.b) {
        uint64_t m = wmin_s[0][tid];
#pragma unroll
        for (int i = 1; i < 8; ++i) m = wmin_s[i][tid] < m ? wmin_s[i][tid] : m;
        p.wgmin[(size_t)tid * p.n_splits + sp] = m;
    }
}

// ---------------------------------------------------------------------------------------
// Per query: T = the R-th smallest of the NB block minima (pairs (ordered key, index), all
// distinct), then the candidate list: exactly R blocks have a minimum <= T and they hold every entry
// whose pair is <= T (at most 32 R, see the file header; `cap` >= that bound), so only those
// blocks' keys are read, 128 bytes each.  One workgroup of 1024 threads per query.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThrThreads) void block_threshold_kernel(const uint64_t *bmin, int64_t nb, int r_sel,
                                                                      const float *keys, int64_t n_pad, int n,
                                                                      uint64_t *cand, int32_t *cand_count, int cap)
{
    __shared__ uint64_t list[kThrList];
    __shared__ uint64_t sel_s;
    __shared__ int list_n;
    __shared__ int blk_n, cnt_s;
    __shared__ int32_t blk_s[kMaxRescore];
    const int q = blockIdx.x, tid = threadIdx.x;
    const uint64_t *bq = bmin + (size_t)q * nb;
    // fewer blocks than wanted entries: everything passes
    const uint64_t t = r_sel >= nb ? kSentinel : rth_smallest_of(bq, nb, r_sel, list, &sel_s, &list_n, tid);
    if (tid == 0) {
        blk_n = 0;
        cnt_s = 0;
    }
    __syncthreads();
    for (int64_t i = tid; i < nb; i += kThrThreads) {
        if (bq[i] <= t) {
            const int pos = atomicAdd(&blk_n, 1);
            if (pos < kMaxRescore) blk_s[pos] = (int32_t)i;
        }
    }
    __syncthreads();
    const int nblk = blk_n < kMaxRescore ? blk_n : kMaxRescore;   // = min(r_sel, nb)
    const float *kq = keys + (size_t)q * n_pad;
    for (int c = tid; c < nblk * 32; c += kThrThreads) {
        const int64_t idx = (int64_t)blk_s[c >> 5] * 32 + (c & 31);
        const uint64_t pr = ((uint64_t)ordered_bits(kq[idx]) << 32) | (uint32_t)idx;
        if (pr <= t && idx < n) {
            const int pos = atomicAdd(&cnt_s, 1);
            if (pos < cap) cand[(size_t)q * cap + pos] = pr;
        }
    }
    __syncthreads();
    if (tid == 0) cand_count[q] = cnt_s;
}

}  // namespace

bool select_supported(int64_t n_pad, int r)
{
    const int64_t nb = n_pad / 32;
    return ((nb + kThrGroups - 1) / kThrGroups) * r <= kThrList;
}

bool skinny_supported(int64_t b, int64_t n_pad, int64_t d_pad, int r, int num_cus)
{
    // The finishing kernel gathers up to r whole groups of block minima into a list of kThrList
    // entries; a group is what one streaming workgroup wrote, and it reads the group minima with
    // one thread each.
    const int64_t n_tiles = n_pad / kTileN;
    const int64_t groups = plan_skinny_splits(n_pad, num_cus);
    const int64_t bpg = ((n_tiles + groups - 1) / groups) * (kTileN / 32);
    return b >= 1 && b <= kSkinnyRows && d_pad <= kSkinnyMaxD && groups <= kThrThreads && bpg * r <= kThrList;
}

size_t select_workspace_bytes(int64_t rows, int64_t n_pad, int r, size_t align)
{
    auto up = [&](size_t x) { return (x + align - 1) / align * align; };
    const size_t b = (size_t)rows;
    return up(b * (size_t)n_pad * 4) + up(b * (size_t)(n_pad / 32) * 8) + up(b * 4) + up(b * (size_t)(32 * r) * 8);
}

int plan_skinny_splits(int64_t n, int num_cus)
{
    const int n_tiles = (int)((n + kTileN - 1) / kTileN);
    const int s = 2 * num_cus < n_tiles ? 2 * num_cus : n_tiles;   // two workgroups per CU
    return s < 1 ? 1 : s;
}

size_t skinny_workspace_bytes(int64_t n_pad, int r, size_t align)
{
    auto up = [&](size_t x) { return (x + align - 1) / align * align; };
    // the block minima and the per-workgroup minima (at most one workgroup per tile)
    return up((size_t)kSkinnyRows * (size_t)(n_pad / 32) * 8) + up((size_t)kSkinnyRows * (size_t)(n_pad / kTileN) * 8) +
           skinny_finish_workspace_bytes(r, align);
}

hipError_t launch_skinny_stream(const SkinnyLaunch &a, hipStream_t s)
{
    if (!a.flag_count || !a.tickets) return hipErrorInvalidValue;
    if (!a.queries || a.d < 1 || a.d > a.d_pad || a.d_pad > kSkinnyMaxD || a.d_pad % kPadD != 0 || a.r < 1 || a.r > kMaxRescore || a.b < 1 || a.b > kSkinnyRows)
        return hipErrorInvalidValue;
    SkinnyArgs k{};
    k.queries = a.queries;
    k.d = a.d;
    k.c_bf = a.c_bf;
    k.norm = a.norm;
    k.mu = a.mu;
    k.bmin = a.bmin;
    k.wgmin = a.wgmin;
    k.flag_count = a.flag_count;
    k.tickets = a.tickets;
    k.b = a.b;
    k.d_pad = a.d_pad;
    k.n_pad = a.n_pad;
    k.n_tiles = (int)(a.n_pad / kTileN);
    k.n_splits = a.n_splits;
    if (a.d_pad <= 512)
        hipLaunchKernelGGL((dist_skinny_kernel<SkinnyCfg<512, 3>>), dim3(a.n_splits), dim3(512), 0, s, k);
    else
        hipLaunchKernelGGL((dist_skinny_kernel<SkinnyCfg<1024, 2>>), dim3(a.n_splits), dim3(512), 0, s, k);
    return hipGetLastError();
}

hipError_t launch_select(const float *keys, const uint64_t *bmin, int64_t n_pad, int n, int b, int r,
                         int32_t *cand_count, uint64_t *cand, hipStream_t s)
{
    const int64_t nb = n_pad / 32;
    if (!select_supported(n_pad, r) || b < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(block_threshold_kernel, dim3(b), dim3(kThrThreads), 0, s, bmin, nb, r, keys, n_pad, n, cand, cand_count,
                       32 * r);
    return hipGetLastError();
}

}  // namespace fz
