// Distance pass of the cache look-up on the matrix cores (gfx950 / CDNA4).
//
// For every query row b and cache entry n it forms the ranking key of the squared
// Euclidean distance  |q - c|^2 = |q|^2 + |c|^2 - 2 q.c  without the per-query
// constant:  key(b, n) = |c_n|^2 - 2 * sum_i Q_bf[b,i] * C_bf[n,i]   (bf16 inputs,
// fp32 accumulation on MFMA), and keeps, per query and per range of cache tiles, the
// R entries with the smallest (key, index).  The score matrix never reaches memory:
// a workgroup owns a 256- (or 128-) query tile, walks a range of 256-entry cache
// tiles, and folds each finished tile into a per-query top-R list held in LDS.
// The exact fp32 distances of these candidates are computed by the finishing kernel.
//
// Paper: Sec. 3 (the look-up computes the k nearest neighbours of the layer output)
// and Sec. 4 "Computational Complexity" (the scan over all cached points is the cost).
//
// Work decomposition: unit = (query tile, split); a split is a contiguous range of
// cache tiles.  Units are numbered so that the workgroups resident on one XCD (block
// id modulo 8) hold neighbouring units, which share query tiles and walk the same
// cache tiles, so that operand re-reads are served by that XCD's L2.
//
// Main loop: the tile is held as 16x16x32 bf16 MFMA accumulators (this shape sustains about a
// tenth more than 32x32x16 on random operands: the chip runs matrix work against its power
// limit, and the shader clock it holds depends on the instruction shape and on the data).
// Two wave layouts: 4 waves (2 x 2), one per SIMD, each owning 128 x 128 in 256 AGPRs (the
// R <= 16 variant: a third fewer fragment reads per MFMA; the MFMAs are issued through inline
// asm so that the accumulators stay in AGPRs and the operands in VGPRs), and 8 waves (2 x 4),
// two per SIMD, each owning (TM*32) x 64 in VGPRs (the other variants).
// Both operands are stored in memory in a tiled, pre-swizzled layout ([row tile][k-block][row]
// [32 elements], see tiled_chunk_offset) whose per-k-step blocks are contiguous and are exactly
// the LDS image, so a stage is filled by a linear copy with LDS-direct 16-byte loads (no VGPR
// staging, fully sequential DRAM access) into a ring of NS stages, all in use.  The chunk
// swizzle makes the ds_read_b128 fragment reads bank-conflict free.  The loads are issued with
// inline asm: the compiler would otherwise order every LDS read behind the outstanding direct
// loads, serialising load and compute.  The loops are software-pipelined by hand, one barrier
// per k-step, loads and fragment reads issued one at a time between MFMAs, with scheduling
// barriers pinning the order (details at each loop).
//
// Epilogue (per tile, in column slabs that reuse the operand LDS): waves write their keys to
// the slab; thread t scans row t, collecting a bit mask of keys not above the row's current
// R-th best, then inserts the survivors into the row's list (keys and entry indices in
// separate LDS arrays) under the total order (key, index).
#include "freeze_internal.h"
#include "select_common.h"

#include <type_traits>

namespace fz {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((address_space(3))) void *lds_void_ptr;

template <int BM_, int BK_, int RMAX_, int NS_, int WN_ = 4, bool B_ONCE_ = false>
struct DistCfg {
    static constexpr int BM = BM_, BN = kTileN, BK = BK_, RMAX = RMAX_;
    static constexpr int NS = NS_;                  // operand stages in LDS, all in use (NS - 1 in flight)
    static constexpr int WM = 2, WN = WN_;          // wave grid: 2 x 4 (8 waves) or 2 x 2 (4 waves)
    static constexpr int NWAVES = WM * WN, THREADS = 64 * NWAVES;
    static constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);   // 32 x 32 blocks per wave (epilogue units)
    static constexpr int AM = 2 * TM, BNB = 2 * TN;                  // 16 x 16 MFMA blocks per wave
    static constexpr int NSUB = BK / kKB;           // k-blocks (of 32 elements) per stage
    static constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    static constexpr int A_BYTES = BM * BK * 2;
    static constexpr int OP_BYTES = NS * STAGE_BYTES;
    static constexpr int NI_A = BM * BK * 2 / 1024 / NWAVES;   // direct-load instructions per wave and stage
    static constexpr int NI_B = BN * BK * 2 / 1024 / NWAVES;
    static_assert(BK % kKB == 0, "a stage is a whole number of k-blocks");
    // slab pass: WNS wave columns at a time
    static constexpr int WNS = (WN >= 4 && BM * 4 * 32 * 4 <= OP_BYTES) ? 4 : ((WN >= 2 && BM * 2 * 32 * 4 <= OP_BYTES) ? 2 : 1);
    static constexpr int SLABW = WNS * 32;          // keys per row in one slab
    static constexpr bool KEYS = (RMAX == 0);       // no fused selection: write every key (small batches)
    // the launch reads every byte of the cache operand exactly once (one query tile): its loads carry
    // the non-temporal hint, so that the stream does not push the query operand, which every
    // workgroup of an XCD re-reads, out of L2
    static constexpr bool B_ONCE = B_ONCE_;
    static constexpr int TOP_BYTES = RMAX * BM * 8;
    static constexpr int LDS_BYTES = OP_BYTES + TOP_BYTES;
    static_assert(BM * SLABW * 4 <= OP_BYTES, "slab must fit in the operand area");
    static_assert(LDS_BYTES <= 163840, "LDS budget");
    static_assert(NI_A >= 1 && NI_B >= 1, "load split");
    static_assert(BM <= THREADS, "one scanning thread per row");
    static constexpr int LPS = NI_A + NI_B;         // direct loads per thread and stage
    static_assert(NS >= 2 && NS <= 6 && (NS - 1) * LPS <= 63, "vmcnt range");
    static_assert(BK == 32, "a k-step is one 16x16x32 MFMA layer");
};

struct DistKernelArgs {
    const uint16_t *q_bf;
    const uint16_t *c_bf;
    const float *norm;
    uint64_t *part;
    const int32_t *count;
    int b, n, d_pad;
    int n_tiles, n_splits, r;
    int alloc_splits, max_splits, num_cus;
    // keys-out variant only:
    float *keys;      // [b_pad, n_pad]
    uint64_t *bmin;   // [b_pad, n_pad / 32]
    int64_t n_pad;
    // stream-K (keys-out variant, one query tile): workgroup x owns k-steps [x sk_len, (x+1) sk_len)
    // of the flattened (cache tile, k-step) space and leaves its accumulators, one slot per tile
    // it touches, in `partial`; 0 = off.
    float *partial;   // [workgroups * sk_slots] slots of BM x BN fp32 in fragment order
    int sk_len, sk_slots;
    // balanced decomposition (fused variants, host-side count): bal_f workgroups per query tile
    // share cache tiles [0, bal_nfull) and the remaining workgroups of the grid share what is
    // left of all query tiles; 0 = off.
    int bal_f, bal_nfull;
    // keys-out variant as a plain projection: out = acc + norm[col] (the bias), optionally through
    // ReLU, no block minima
    int projection, relu;
};

// Epilogue of the keys-out variant: every key of the tile and the minimum of every block of 32
// entries.  Keys pass through the LDS slab so that the global stores are whole 512-byte row pieces.
template <class C>
__device__ __forceinline__ void keys_epilogue(f32x4 (&acc)[C::AM][C::BNB], const DistKernelArgs &p, float *slab, int mt,
                                              int n0, int nq, int w, int wm, int wn, int lane)
{
    constexpr int BM = C::BM, TM = C::TM, TN = C::TN;
    const float scale = p.projection ? 1.f : -2.f;
    static_assert(!C::KEYS || C::WNS == C::WN, "keys-out epilogue: one slab pass covers all wave columns");
#pragma unroll
    for (int bj = 0; bj < TN; ++bj) {
        // the wave's 32 columns of this pass are two MFMA blocks; a lane holds column (lane & 15)
        // of each and rows 4 (lane >> 4) .. + 3 of every 16-row block
#pragma unroll
        for (int v2 = 0; v2 < 2; ++v2) {
            const int col = n0 + wn * TN * 32 + bj * 32 + v2 * 16 + (lane & 15);
            const float nrm = p.norm[col];   // col < n_pad always
            const int sc = wn * 32 + v2 * 16 + (lane & 15);
            // the column swizzle depends on the row modulo NGS = SLABW / 4 only, so the 16-row blocks one
            // period apart share an address up to a constant (an immediate offset)
            constexpr int NGS = C::SLABW / 4, RP = NGS > 16 ? NGS / 16 : 1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
#pragma unroll
                for (int par = 0; par < RP; ++par) {
                    const int row0 = wm * TM * 32 + par * 16 + (lane >> 4) * 4 + e;
                    float *dst = slab + row0 * C::SLABW + ((((sc >> 2) ^ row0) & (NGS - 1)) << 2) + (sc & 3);
#pragma unroll
                    for (int bi = par; bi < C::AM; bi += RP) {
                        float v = __builtin_fmaf(scale, acc[bi][2 * bj + v2][e], nrm);
                        if (p.relu) v = __builtin_fmaxf(v, 0.f);
                        dst[(bi - par) * 16 * C::SLABW] = v;
                    }
                }
            }
        }
        __syncthreads();
        // a row of the slab is LPR lanes x 4 keys; a wave copies 64 / LPR rows per round
        constexpr int LPR = C::SLABW / 4, RPW = 64 / LPR;
        const int lr = lane % LPR;
        const int seg = lr >> 3;                                   // wave column the 4 keys came from
        const int gcol = n0 + seg * TN * 32 + bj * 32 + (lr & 7) * 4;   // entry index of the first key
#pragma unroll 2
        for (int it = 0; it < BM / (RPW * C::NWAVES); ++it) {
            const int row = (it * C::NWAVES + w) * RPW + lane / LPR;
            const int grow = mt * BM + row;
            const f32x4 v = reinterpret_cast<const f32x4 *>(slab + row * C::SLABW)[(lr ^ row) & (LPR - 1)];
            const bool live = grow < nq;
            if (live) *reinterpret_cast<f32x4 *>(p.keys + (size_t)grow * p.n_pad + gcol) = v;
            // minimum (key, index) pair of the 32-entry block: 4 own keys, then the 8 lanes of the block
            uint64_t mn = ((uint64_t)ordered_bits(v[0]) << 32) | (uint32_t)gcol;
#pragma unroll
            for (int e = 1; e < 4; ++e) {
                const uint64_t pr = ((uint64_t)ordered_bits(v[e]) << 32) | (uint32_t)(gcol + e);
                mn = pr < mn ? pr : mn;
            }
#pragma unroll
            for (int off = 4; off >= 1; off >>= 1) {
                const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)mn, off, 64);
                const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(mn >> 32), off, 64);
                const uint64_t o = ((uint64_t)hi << 32) | lo;
                mn = o < mn ? o : mn;
            }
            if (live && (lr & 7) == 0 && !p.projection) p.bmin[(size_t)grow * (p.n_pad / 32) + (gcol >> 5)] = mn;
        }
        __syncthreads();
    }
}

template <class C>
__global__ __launch_bounds__(C::THREADS) void dist_topr_kernel(DistKernelArgs p)
{
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, TM = C::TM, TN = C::TN;
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::LDS_BYTES];
    // Per-row candidate lists: keys (ordered bits) in chunks of four slots, [RMAX / 4][BM][4], so that
    // a row's thread reads its whole list with RMAX / 4 conflict-free 16-byte reads; entry indices [RMAX][BM].
    uint32_t *top_key = reinterpret_cast<uint32_t *>(smem + C::OP_BYTES);
    uint32_t *top_idx = top_key + C::RMAX * BM;
    auto key_slot = [&](int i, int t) { return ((i >> 2) * BM + t) * 4 + (i & 3); };
    float *slab = reinterpret_cast<float *>(smem);                      // [BM][SLABW], aliases operands
    const bf16x8 *smem16 = reinterpret_cast<const bf16x8 *>(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w / C::WN, wn = w % C::WN;

    // How many query tiles are live decides the number of splits (on the device when the count
    // lives there); workgroups beyond live tiles x splits have nothing to do.
    const int nq = p.count ? *p.count : p.b;
    const int live_mt = (nq + BM - 1) / BM;
    const int n_splits = p.count ? splits_for(live_mt, p.n_tiles, p.num_cus, p.max_splits) : p.n_splits;
    const bool stream_k = C::KEYS && p.sk_len > 0;
    const bool balanced = !C::KEYS && p.bal_f > 0;
    const int units = stream_k ? (int)gridDim.x : (balanced ? live_mt * p.bal_f : live_mt * n_splits);
    if (!balanced && (int)blockIdx.x >= units) return;   // uniform per workgroup, before any barrier
    // XCD-aware unit numbering: blocks with equal (id % 8) run on one XCD; give them a contiguous
    // range of units.  units = 8a + rem: XCD x owns a (+1 if x < rem) consecutive units.
    int unit;
    {
        const int a = units >> 3, rem = units & 7;
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
        unit = x * a + (x < rem ? x : rem) + j;
    }
    const int r = p.r;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void_ptr)smem;
    const size_t tile_row_bytes = (size_t)p.d_pad * 2;   // bytes of one row; a tile of T rows holds T * this
    const uint32_t lane_off = w * 1024 + lane * 16;

    // A workgroup handles one part (query tile, range of cache tiles, output list slot), except
    // under the balanced decomposition: there bal_f workgroups per query tile cut cache tiles
    // [0, bal_nfull) evenly, and the grid's remaining workgroups cut the flattened remainder
    // (query tile, cache tile >= bal_nfull) evenly, so that one of them may serve the tail of one
    // query tile and the head of the next.  A query tile's remainder lies in at most two of them:
    // the first writes list slot bal_f, the second bal_f + 1 (filled with "no entry" by the first
    // when there is no second).
    const int w_full = live_mt * p.bal_f;
    const int lo = p.n_tiles - p.bal_nfull;   // remainder tiles per query tile (balanced only)
    int rem_c = 0, rem_end = 0;               // this workgroup's range of the flattened remainder
    if (balanced && (int)blockIdx.x >= w_full) {
        const int64_t total_lo = (int64_t)live_mt * lo;
        const int lw = (int)gridDim.x - w_full, i = (int)blockIdx.x - w_full;
        rem_c = (int)(total_lo * i / lw);
        rem_end = (int)(total_lo * (i + 1) / lw);
    }
    bool first_part = true;
    while (true) {
        int mt, nt0, nt1, slot;
        bool clear_next_slot = false;
        if (balanced && (int)blockIdx.x >= w_full) {
            if (rem_c >= rem_end) break;
            mt = rem_c / lo;
            const int off = rem_c - mt * lo;
            const int len = (lo - off < rem_end - rem_c) ? lo - off : rem_end - rem_c;
            nt0 = p.bal_nfull + off;
            nt1 = nt0 + len;
            slot = p.bal_f + (off == 0 ? 0 : 1);
            clear_next_slot = (off == 0 && len == lo);
            rem_c += len;
        } else {
            if (!first_part) break;
            if (balanced) {
                mt = unit / p.bal_f;
                slot = unit % p.bal_f;
                nt0 = (int)(((int64_t)slot * p.bal_nfull) / p.bal_f);
                nt1 = (int)(((int64_t)(slot + 1) * p.bal_nfull) / p.bal_f);
            } else {
                mt = stream_k ? 0 : unit / n_splits;
                slot = stream_k ? 0 : unit % n_splits;
                nt0 = (int)(((int64_t)slot * p.n_tiles) / n_splits);
                nt1 = (int)(((int64_t)(slot + 1) * p.n_tiles) / n_splits);
            }
        }
        first_part = false;

        // per-row selection state lives with thread t (< BM)
        // kmax = key of the list's largest entry under the order (key, index), held in slot maxpos (its
        // index is looked up only when a key equal to kmax turns up); slots past r hold the smallest key
        // and never count
        uint32_t kmax = 0xffffffffu;
        int maxpos = 0;
        int fill = 0;   // slots taken while the list still has empty ones (they fill in order)
        float tau = __builtin_inff();
        if constexpr (!C::KEYS) {
            if (tid < BM) {
#pragma unroll
                for (int i = 0; i < C::RMAX; ++i) {
                    top_key[key_slot(i, tid)] = i < p.r ? 0xffffffffu : 0u;
                    top_idx[i * BM + tid] = 0xffffffffu;
                }
            }
        }

        // Direct loads copy a stage linearly: wave w, instruction i moves the 1 KiB at offset
        // (i * NWAVES + w) * 1024 of the stage's A (or B) image; lane l moves 16 bytes at + 16 l.
        const uint64_t gA_part = uniform_u64((uint64_t)(uintptr_t)p.q_bf + (size_t)mt * BM * tile_row_bytes);
        // fragment read addresses, in 16-byte units relative to the stage's A / B image
        // (a 16x16x32 operand: lane l holds row l & 15 of the block and the 8 elements of chunk l >> 4;
        // rows 16 apart share their swizzle)
        const int rowA = wm * TM * 32 + (lane & 15);
        const int rowB = wn * TN * 32 + (lane & 15);
        const int rdA = rowA * 4 + ((lane >> 4) ^ tiled_chunk_swizzle(rowA));
        const int rdB = rowB * 4 + ((lane >> 4) ^ tiled_chunk_swizzle(rowB));
        const int nk = p.d_pad / BK;

        // The workgroup walks segments (cache tile, range of k-steps) of the flattened space: whole
        // tiles nt0 .. nt1-1, or under stream-K the k-steps [x sk_len, (x+1) sk_len) whatever tiles
        // they fall in.  Segment s of the range lies in tile (first tile + s); that number also names
        // the slot its accumulators are left in, whatever order the segments are taken in.
        // Under stream-K a range that ends inside a tile is taken with that last piece (k-steps from
        // 0 up) first: then every workgroup moves through the depth upwards from 0, skipping one
        // gap, and at any moment the workgroups of the chip read the query operand at two places
        // of the depth instead of one place per starting offset, so most of those reads hit in L2.
        const int64_t sk_total = (int64_t)live_mt * p.n_tiles * nk;   // stream-K: (query tile, cache tile, k-step)
        const int64_t g_begin = stream_k ? (int64_t)blockIdx.x * p.sk_len : (int64_t)nt0 * nk;
        const int64_t g_end = stream_k ? ((int64_t)(blockIdx.x + 1) * p.sk_len < sk_total
                                              ? (int64_t)(blockIdx.x + 1) * p.sk_len
                                              : sk_total)
                                       : (int64_t)nt1 * nk;
        const int tile0 = (int)(g_begin / nk);
        const int nseg = g_begin < g_end ? (int)((g_end - 1) / nk) - tile0 + 1 : 0;
        const bool head_first = stream_k && nseg >= 2 && g_end < (int64_t)(tile0 + nseg) * nk;
        // 4-wave fused variant: the first stages of a part's next tile are requested before the
        // epilogue of the current one (whose slab leaves the upper stages alone) and land during it
        constexpr int PF = (!C::KEYS && C::WN == 2) ? (C::OP_BYTES - BM * C::SLABW * 4) / C::STAGE_BYTES : 0;
        static_assert(PF >= 0 && PF < C::NS, "prefetched stages lie above the slab");
        bool prefetched = false;
        for (int it = 0; it < nseg; ++it) {
            const int seg = head_first ? (it == 0 ? nseg - 1 : it - 1) : it;
            const int tile = tile0 + seg;                     // under stream-K: query tile * n_tiles + cache tile
            const int nt = stream_k ? tile % p.n_tiles : tile;
            const int smt = stream_k ? tile / p.n_tiles : mt;   // the segment's query tile
            const int ka = seg == 0 ? (int)(g_begin - (int64_t)tile0 * nk) : 0;                // first k-step of the segment
            const int kb = seg == nseg - 1 ? (int)(g_end - (int64_t)tile * nk) : nk;          // one past its last
            const int n0 = nt * BN;
            const uint64_t gA = stream_k
                                    ? uniform_u64((uint64_t)(uintptr_t)p.q_bf + (size_t)smt * BM * tile_row_bytes)
                                    : gA_part;
            const uint64_t gB = uniform_u64((uint64_t)(uintptr_t)p.c_bf + (size_t)nt * BN * tile_row_bytes);
            // one instruction of a stage's fill: l < NI_A -> A image, else B image
            auto issue_one = [&](int stage, int kt, int l) {
                const uint32_t sbase = smem_base + stage * C::STAGE_BYTES + w * 1024;
                if (l < C::NI_A)
                    load16_global_to_lds(gA + (size_t)kt * C::A_BYTES + l * (C::NWAVES * 1024), lane_off,
                                         sbase + l * (C::NWAVES * 1024));
                else if constexpr (C::B_ONCE)
                    load16_global_to_lds_nt(gB + (size_t)kt * (BN * BK * 2) + (l - C::NI_A) * (C::NWAVES * 1024), lane_off,
                                         sbase + C::A_BYTES + (l - C::NI_A) * (C::NWAVES * 1024));
                else
                    load16_global_to_lds(gB + (size_t)kt * (BN * BK * 2) + (l - C::NI_A) * (C::NWAVES * 1024), lane_off,
                                         sbase + C::A_BYTES + (l - C::NI_A) * (C::NWAVES * 1024));
            };

            f32x4 acc[C::AM][C::BNB];
#pragma unroll
            for (int i = 0; i < C::AM; ++i)
#pragma unroll
                for (int j = 0; j < C::BNB; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

            {
                if constexpr (C::WN == 2) {
                    // ---- one wave per SIMD: 128 x 128 per wave, accumulators in AGPRs ----
                    // All NS stages are in use: at the top of k-step kt its fragments are in (or on their
                    // way to) register buffer kt & 1, k-block kt+1 has landed, kt+2 .. kt+NS-1 are in
                    // flight.  The step's barrier (after the wave's own loads of kt+1 and its own reads of
                    // kt are done) publishes kt+1 and frees the stage of kt, which is refilled with kt+NS
                    // during the step.  With a single wave on the SIMD nothing else covers an issue stall,
                    // so every memory instruction goes alone into the shadow of an MFMA (the pipe is busy
                    // 16 cycles per MFMA, issuing one takes 4), and the next step's fragment reads all
                    // leave during the first 48 MFMAs, so that the wait for them at the next top is free.
                    // The compiler does not know these MFMAs: the waits that order them against the LDS
                    // reads are the explicit ones here, and the no-ops after the loop cover the distance
                    // the hardware wants between the last MFMA and the first read of an accumulator.
                    constexpr int AMB = C::AM, BB = C::BNB;   // 8 x 8 blocks
                    static_assert(AMB == 8 && BB == 8, "4-wave loop is written for 128 x 128 per wave");
                    // k-block ka + ps goes to stage (s0 + ps) % NS; a prefetched tile starts in the first
                    // stage above the slab and has its first PF stages on their way already
                    const int s0 = prefetched ? C::NS - PF : 0;
#pragma unroll
                    for (int ps = 0; ps < C::NS; ++ps) {
                        if (ps < PF && prefetched) continue;
                        const int stg = s0 + ps < C::NS ? s0 + ps : s0 + ps - C::NS;
#pragma unroll
                        for (int l = 0; l < C::LPS; ++l) issue_one(stg, ka + ps < kb ? ka + ps : kb - 1, l);
                    }
                    wait_global_loads_le<(C::NS - 1) * C::LPS>();
                    __syncthreads();
                    bf16x8 af[2][AMB], bfr[2][BB];
                    auto read_a = [&](int buf, int stage, int i) { af[buf][i] = smem16[stage * (C::STAGE_BYTES / 16) + rdA + i * 64]; };
                    auto read_b = [&](int buf, int stage, int j) { bfr[buf][j] = smem16[stage * (C::STAGE_BYTES / 16) + C::A_BYTES / 16 + rdB + j * 64]; };
#pragma unroll
                    for (int j = 0; j < BB; ++j) read_b(0, s0, j);
#pragma unroll
                    for (int i = 0; i < AMB; ++i) read_a(0, s0, i);
                    int st = s0;
                    auto k_step = [&](int kt, auto buf_tag) {
                        constexpr int buf = decltype(buf_tag)::value;
                        const int nst = (st + 1 == C::NS) ? 0 : st + 1;
                        const int fill_kt = kt + C::NS < kb ? kt + C::NS : kb - 1;
                        // own part of k-block kt+1 has landed; own reads of k-block kt are done
                        wait_global_loads_le<(C::NS - 2) * C::LPS>();
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        __syncthreads();   // k-block kt+1 is everyone's; stage st is free
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < AMB; ++i) {
#pragma unroll
                            for (int j = 0; j < BB; ++j) {
                                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(af[buf][i]), "v"(bfr[buf][j]));
                                __builtin_amdgcn_sched_barrier(0);
                                // one memory instruction at a time in the shadow of an MFMA: the next k-block's
                                // fragments (B blocks, then A blocks) after every third MFMA of the first 48, a
                                // refill load after every eighth
                                constexpr int RD_EVERY = 3;
                                const int slot = i * BB + j;
                                if (slot % RD_EVERY == 1 && slot / RD_EVERY < AMB + BB) {
                                    const int rr = slot / RD_EVERY;
                                    if (rr < BB) read_b(buf ^ 1, nst, rr);
                                    else read_a(buf ^ 1, nst, rr - BB);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                                if (slot % 8 == 6) {
                                    issue_one(st, fill_kt, slot / 8);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                            }
                        }
                        st = nst;
                    };
                    for (int kt = ka; kt < kb; kt += 2) {
                        k_step(kt, std::integral_constant<int, 0>{});
                        k_step(kt + 1, std::integral_constant<int, 1>{});
                    }
                    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");   // MFMA results before the accumulators are read
                } else {
                    // Software-pipelined loop.  A k-step is one MFMA layer (32 deep), taken in two halves:
                    // the wave's upper A blocks against all its B blocks, then the lower ones.  Invariant at
                    // the top of k-step kt: its first A half and its B blocks are in (or on their way to)
                    // registers; k-blocks kt+1 .. kt+NS-1 are in flight or landed in the other stages.  The
                    // second A half is read during the first half's MFMAs; after that every read of the
                    // current stage has been issued, so the step's only barrier goes there: it publishes the
                    // next stage (each wave waited for its own part) and frees the current one.  The MFMAs of
                    // the second half need nothing newer, so the matrix pipe restarts at once, and the next
                    // stage's first fragments and the refill of the freed stage are issued one by one between
                    // them: a wave blocks while the memory pipeline accepts a load, so loads issued back to
                    // back stall the MFMAs behind them.  Past the last k-block the refills repeat it (never
                    // read): the loop body and the count of outstanding loads stay uniform.  B fragments
                    // alternate between two register sets from one k-step to the next, so the loop takes
                    // k-steps in pairs (every range of k-steps here has an even length).
                    constexpr int KS = 2;                  // halves of a k-step
                    constexpr int AH = C::AM / 2;          // A blocks (MFMA groups of BNB) per half
                    constexpr int NR1 = AH + C::BNB;       // fragment reads issued during the second half
                    // A stage's LPS loads are issued in two parts: LB of them between the MFMAs of the second
                    // half of the k-step that frees the stage, the rest between the MFMAs of the following
                    // k-step's first half, so that loads leave at an even rate.
                    constexpr int LB = C::LPS / KS;
                    constexpr int G1 = AH;                 // MFMA groups before the barrier
#pragma unroll
                    for (int ps = 0; ps < C::NS; ++ps)
#pragma unroll
                        for (int l = 0; l < (ps == C::NS - 1 ? LB : C::LPS); ++l) issue_one(ps, ka + ps < kb ? ka + ps : kb - 1, l);
                    wait_global_loads_le<(C::NS - 2) * C::LPS + LB>();
                    __syncthreads();
                    bf16x8 af[2][AH], bfr[2][C::BNB];
                    auto read_a = [&](int h, int stage, int i) {   // A block h * AH + i of the stage
                        af[h][i] = smem16[stage * (C::STAGE_BYTES / 16) + rdA + (h * AH + i) * 64];
                    };
                    auto read_b = [&](int set, int stage, int j) {
                        bfr[set][j] = smem16[stage * (C::STAGE_BYTES / 16) + C::A_BYTES / 16 + rdB + j * 64];
                    };
#pragma unroll
                    for (int i = 0; i < AH; ++i) read_a(0, 0, i);
#pragma unroll
                    for (int j = 0; j < C::BNB; ++j) read_b(0, 0, j);
                    int st = 0;
                    auto k_step = [&](int kt, auto set_tag) {
                        constexpr int set = decltype(set_tag)::value;   // B register set of this k-step
                        const int nst = (st + 1 == C::NS) ? 0 : st + 1;
                        const int pst = (st == 0) ? C::NS - 1 : st - 1;
                        const int fill_kt = kt + C::NS < kb ? kt + C::NS : kb - 1;
                        const int pfill_kt = kt + C::NS - 1 < kb ? kt + C::NS - 1 : kb - 1;   // the stage freed one step ago
#pragma unroll
                        for (int i = 0; i < AH; ++i) read_a(1, st, i);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < AH; ++i) {
#pragma unroll
                            for (int j = 0; j < C::BNB; ++j)
                                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[0][i], bfr[set][j], acc[i][j], 0, 0, 0);
                            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                            for (int l = LB + i * (C::LPS - LB) / G1; l < LB + (i + 1) * (C::LPS - LB) / G1; ++l)
                                issue_one(pst, pfill_kt, l);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        wait_global_loads_le<(C::NS - 2) * C::LPS>();   // own part of k-block kt+1 has landed
                        __syncthreads();                                // ... everyone's; and stage st is free
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < AH; ++i) {
#pragma unroll
                            for (int j = 0; j < C::BNB; ++j)
                                acc[AH + i][j] =
                                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[1][i], bfr[set][j], acc[AH + i][j], 0, 0, 0);
                            constexpr int RG = AH > 1 ? AH - 1 : 1;   // the reads go with the first AH-1 groups
#pragma unroll
                            for (int rr = i * NR1 / RG; rr < (i + 1) * NR1 / RG && rr < NR1 && i < RG; ++rr) {
                                if (rr < AH)
                                    read_a(0, nst, rr);
                                else
                                    read_b(set ^ 1, nst, rr - AH);
                            }
                            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                            for (int l = i * LB / AH; l < (i + 1) * LB / AH; ++l) issue_one(st, fill_kt, l);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        st = nst;
                    };
                    for (int kt = ka; kt < kb; kt += 2) {
                        k_step(kt, std::integral_constant<int, 0>{});
                        k_step(kt + 1, std::integral_constant<int, 1>{});
                    }
                }
                wait_global_loads_le<0>();   // the refills past the last k-block
            }
            __syncthreads();   // operand LDS is free: the slab may overwrite it

            if constexpr (C::KEYS) {
                if (p.sk_len > 0) {
                    // stream-K: leave the accumulators of this (tile, k-range) in the workgroup's next slot
                    f32x4 *dst = reinterpret_cast<f32x4 *>(p.partial) +
                                 ((size_t)blockIdx.x * p.sk_slots + seg) * (size_t)(BM * BN / 4);
#pragma unroll
                    for (int bi = 0; bi < C::AM; ++bi)
#pragma unroll
                        for (int bj = 0; bj < C::BNB; ++bj) dst[((w * C::AM + bi) * C::BNB + bj) * 64 + lane] = acc[bi][bj];
                    continue;
                }
                keys_epilogue<C>(acc, p, slab, smt, n0, nq, w, wm, wn, lane);
                continue;
            }
            // ---- epilogue: fold this tile into the per-row top-R lists ----
            // The norms of the wave's columns are fetched first: nothing else in the epilogue loads from
            // memory, so the prefetch below is never part of a wait.
            // (the lane number is made opaque here: addresses derived from it are then recomputed per tile
            // instead of being kept, and spilled, across the main loop)
            int elane = lane;
            asm volatile("" : "+v"(elane));
            float nrm_r[C::BNB];
#pragma unroll
            for (int cb = 0; cb < C::BNB; ++cb) nrm_r[cb] = p.norm[n0 + wn * TN * 32 + cb * 16 + (elane & 15)];   // < n_pad always
            if constexpr (PF > 0) {
                prefetched = false;
                // the norms are in registers by here (the compiler places its waits for them in front of
                // this) and cannot be fetched again later
#pragma unroll
                for (int cb = 0; cb < C::BNB; ++cb) asm volatile("" : "+v"(nrm_r[cb]));
                if (it + 1 < nseg) {   // uniform; fused variants walk whole tiles in order: the next one is nt + 1
                    const uint64_t gBn = uniform_u64((uint64_t)(uintptr_t)p.c_bf + (size_t)(nt + 1) * BN * tile_row_bytes);
#pragma unroll
                    for (int ps = 0; ps < PF; ++ps)
#pragma unroll
                        for (int l = 0; l < C::LPS; ++l) {
                            const uint32_t sbase = smem_base + (C::NS - PF + ps) * C::STAGE_BYTES + w * 1024;
                            if (l < C::NI_A)
                                load16_global_to_lds(gA + (size_t)ps * C::A_BYTES + l * (C::NWAVES * 1024), lane_off,
                                                     sbase + l * (C::NWAVES * 1024));
                            else
                                load16_global_to_lds(gBn + (size_t)ps * (BN * BK * 2) + (l - C::NI_A) * (C::NWAVES * 1024), lane_off,
                                                     sbase + C::A_BYTES + (l - C::NI_A) * (C::NWAVES * 1024));
                        }
                    prefetched = true;
                }
            }
#pragma unroll
            for (int bj = 0; bj < TN; ++bj) {
#pragma unroll 1
                for (int wg = 0; wg < C::WN / C::WNS; ++wg) {
                    if (wn / C::WNS == wg) {
                        // the wave's 32 columns of this pass are two MFMA blocks; a lane holds column
                        // (lane & 15) of each and rows 4 (lane >> 4) .. + 3 of every 16-row block
#pragma unroll
                        for (int v2 = 0; v2 < 2; ++v2) {
                            const float nrm = nrm_r[2 * bj + v2];
                            const int sc = (wn % C::WNS) * 32 + v2 * 16 + (elane & 15);
                            // the column swizzle depends on the row modulo NGS = SLABW / 4 only, so the 16-row
                            // blocks one period apart share an address up to a constant (an immediate offset)
                            constexpr int NGS = C::SLABW / 4, RP = NGS > 16 ? NGS / 16 : 1;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
#pragma unroll
                                for (int par = 0; par < RP; ++par) {
                                    const int row0 = wm * TM * 32 + par * 16 + (elane >> 4) * 4 + e;
                                    float *dst = slab + row0 * C::SLABW + ((((sc >> 2) ^ row0) & (NGS - 1)) << 2) + (sc & 3);
#pragma unroll
                                    for (int bi = par; bi < C::AM; bi += RP)
                                        dst[(bi - par) * 16 * C::SLABW] = __builtin_fmaf(-2.f, acc[bi][2 * bj + v2][e], nrm);
                                }
                            }
                        }
                    }
                    __syncthreads();
                    if (tid < BM) {
                        int t = tid;
                        asm volatile("" : "+v"(t));   // opaque: slab addresses are recomputed here, not kept across the main loop
                        // First pass over the row: one bit per group of four columns whose smallest key
                        // is not above the row's current R-th best (two min instructions and a compare
                        // per four keys); almost every group fails once the list has filled.
                        const f32x4 *srow = reinterpret_cast<const f32x4 *>(slab + t * C::SLABW);
                        constexpr int NG = C::SLABW / 4;
                        static_assert(NG <= 32, "one mask word");
                        // (sixteen groups are read before the first is looked at, so that the reads overlap;
                        // the minima go through v_min3_f32 directly: the keys are never NaN)
                        uint32_t gmask = 0;
#pragma unroll
                        for (int c0 = 0; c0 < NG; c0 += 16) {
                            f32x4 v[16];
#pragma unroll
                            for (int c = 0; c < 16; ++c) v[c] = srow[((c0 + c) ^ t) & (NG - 1)];
#pragma unroll
                            for (int c = 0; c < 16; ++c) {
                                float m;
                                asm("v_min3_f32 %0, %1, %2, %3" : "=v"(m) : "v"(v[c][0]), "v"(v[c][1]), "v"(v[c][2]));
                                asm("v_min_f32 %0, %1, %2" : "=v"(m) : "v"(m), "v"(v[c][3]));
                                gmask |= (uint32_t)(m <= tau) << (c0 + c);
                            }
                        }
                        // Second pass: the flagged groups give a bit per key that passes and is a real
                        // cache entry (padding columns are not).
                        uint64_t kmask[2] = {0, 0};
                        while (gmask) {
                            const int cg = __builtin_ctz(gmask);
                            gmask &= gmask - 1;
                            const f32x4 v = srow[(cg ^ t) & (NG - 1)];
                            // the four keys share a 32-column segment: columns seg0 .. seg0+3 of the tile
                            const int seg0 = (wg * C::WNS + (cg >> 3)) * TN * 32 + bj * 32 + ((cg & 7) << 2);
                            const int lim = p.n - n0 - seg0;   // real cache entries iff e < lim
                            uint64_t bits = 0;
#pragma unroll
                            for (int e = 0; e < 4; ++e) bits |= (uint64_t)((v[e] <= tau) && (e < lim)) << e;
                            bits <<= (cg & 15) * 4;
                            if (cg < 16)
                                kmask[0] |= bits;
                            else
                                kmask[1] |= bits;
                        }
                        // Third pass: one insertion attempt per surviving key, against the threshold as it tightens.
#pragma unroll
                        for (int m = 0; m < (NG + 15) / 16; ++m) {
                            uint64_t mk = kmask[m];
                            while (mk) {
                                const int sc = m * 64 + __builtin_ctzll(mk);
                                mk &= mk - 1;
                                const float key = slab[t * C::SLABW + ((((sc >> 2) ^ t) & (NG - 1)) << 2) + (sc & 3)];
                                const int tilecol = (wg * C::WNS + sc / 32) * TN * 32 + bj * 32 + (sc & 31);
                                const uint32_t kb = ordered_bits(key), col = (uint32_t)(n0 + tilecol);
                                if (kb < kmax || (kb == kmax && col < top_idx[maxpos * BM + t])) {
                                    // replace the largest entry, then find the new largest: the largest key, and
                                    // among equal keys (rare) the largest index
                                    top_key[key_slot(maxpos, t)] = kb;
                                    top_idx[maxpos * BM + t] = col;
                                    if (fill + 1 < r) {
                                        // empty slots remain: each of them is a largest entry, the next one
                                        // is taken next, and nothing else about the list's maximum changes
                                        maxpos = ++fill;
                                        continue;
                                    }
                                    fill = r;
                                    u32x4 k4[C::RMAX > 0 ? C::RMAX / 4 : 1];   // (the keys-out variant never gets here)
#pragma unroll
                                    for (int j = 0; j < C::RMAX / 4; ++j)
                                        k4[j] = *reinterpret_cast<const u32x4 *>(top_key + (j * BM + t) * 4);
                                    uint32_t km = 0;
#pragma unroll
                                    for (int i = 0; i < C::RMAX; ++i) km = k4[i >> 2][i & 3] > km ? k4[i >> 2][i & 3] : km;
                                    int pos = 0, same = 0;
#pragma unroll
                                    for (int i = 0; i < C::RMAX; ++i) {
                                        const bool eq = k4[i >> 2][i & 3] == km;
                                        pos = eq ? i : pos;
                                        same += eq;
                                    }
                                    if (same > 1) {
                                        uint32_t im = top_idx[pos * BM + t];
#pragma unroll 1
                                        for (int i = 0; i < r; ++i) {
                                            if (top_key[key_slot(i, t)] == km) {
                                                const uint32_t u = top_idx[i * BM + t];
                                                if (u >= im) { im = u; pos = i; }
                                            }
                                        }
                                    }
                                    kmax = km;
                                    maxpos = pos;
                                    tau = (km == 0xffffffffu) ? __builtin_inff() : from_ordered_bits(km);
                                }
                            }
                        }
                    }
                    __syncthreads();
                }
            }
        }

        if (!C::KEYS && tid < BM) {
            uint64_t *dst = p.part + (((size_t)mt * BM + tid) * p.alloc_splits + slot) * r;
#pragma unroll
            for (int i = 0; i < C::RMAX; ++i)
                if (i < r) {
                    dst[i] = ((uint64_t)top_key[key_slot(i, tid)] << 32) | top_idx[i * BM + tid];
                    if (clear_next_slot) dst[r + i] = kSentinel;
                }
        }
    }   // parts
}

// Stream-K second pass (keys-out variant): per cache tile, add up the accumulators the
// workgroups of the first pass left for it (in workgroup order: a fixed order of additions), then
// the usual epilogue.  One workgroup per tile, same wave layout as the first pass.
template <class C>
__global__ __launch_bounds__(C::THREADS) void keys_fixup_kernel(DistKernelArgs p)
{
    constexpr int BM = C::BM, BN = C::BN;
    __shared__ __attribute__((aligned(16))) unsigned char smem[BM * C::SLABW * 4];
    float *slab = reinterpret_cast<float *>(smem);
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w / C::WN, wn = w % C::WN;
    const int tile = blockIdx.x;                       // query tile * n_tiles + cache tile
    const int nt = tile % p.n_tiles, mt = tile / p.n_tiles;
    const int nk = p.d_pad / C::BK;
    const int64_t g0 = (int64_t)tile * nk, g1 = g0 + nk;
    const int w_first = (int)(g0 / p.sk_len), w_last = (int)((g1 - 1) / p.sk_len);
    f32x4 acc[C::AM][C::BNB];
#pragma unroll
    for (int i = 0; i < C::AM; ++i)
#pragma unroll
        for (int j = 0; j < C::BNB; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    for (int x = w_first; x <= w_last; ++x) {
        const int seg = tile - (int)(((int64_t)x * p.sk_len) / nk);   // tiles workgroup x touched before this one
        const f32x4 *src = reinterpret_cast<const f32x4 *>(p.partial) + ((size_t)x * p.sk_slots + seg) * (size_t)(BM * BN / 4);
#pragma unroll
        for (int bi = 0; bi < C::AM; ++bi)
#pragma unroll
            for (int bj = 0; bj < C::BNB; ++bj) {
                const f32x4 v = src[((w * C::AM + bi) * C::BNB + bj) * 64 + lane];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[bi][bj][e] += v[e];
            }
    }
    const int nq = p.count ? *p.count : p.b;
    keys_epilogue<C>(acc, p, slab, mt, nt * BN, nq, w, wm, wn, lane);
}

DistPlan plan_dist(int64_t b, int64_t n, int r, int num_cus, bool keys_out, int64_t d_pad)
{
    DistPlan pl{};
    pl.variant = keys_out ? 3 : (r <= 16 ? 0 : (r <= 32 ? 1 : 2));
    pl.bm = pl.variant == 2 ? 128 : 256;
    pl.r = r;
    pl.m_tiles = (int)((b + pl.bm - 1) / pl.bm);
    if (pl.m_tiles < 1) pl.m_tiles = 1;
    pl.n_tiles = (int)((n + kTileN - 1) / kTileN);
    pl.b_pad = (int64_t)pl.m_tiles * pl.bm;
    pl.num_cus = num_cus;
    pl.max_splits = keys_out ? pl.n_tiles : kMaxMergeEntries / r;
    pl.n_splits = splits_for(pl.m_tiles, pl.n_tiles, num_cus, pl.max_splits);
    // a cascade may run this plan with any live count from 1 tile to all of them
    pl.alloc_splits = pl.n_splits;
    pl.grid_units = pl.m_tiles * pl.n_splits;
    for (int live = 1; live < pl.m_tiles; ++live) {
        const int s = splits_for(live, pl.n_tiles, num_cus, pl.max_splits);
        if (s > pl.alloc_splits) pl.alloc_splits = s;
        if (live * s > pl.grid_units) pl.grid_units = live * s;
    }
    // Balanced decomposition: with s equal splits per query tile the slowest workgroup has
    // ceil(n_tiles / s) tiles and m_tiles * s of the CUs work; cutting the flattened space evenly
    // over all CUs brings that down to about m_tiles * n_tiles / CUs + 1.
    pl.bal_f = pl.bal_nfull = pl.bal_wgs = pl.bal_lists = 0;
    if (!keys_out && pl.m_tiles <= num_cus && (int64_t)pl.m_tiles * pl.n_tiles >= 4 * (int64_t)num_cus) {
        const int f = num_cus / pl.m_tiles;
        const int lw = num_cus - f * pl.m_tiles;
        if (lw > 0 && f + 2 <= pl.max_splits) {
            // tiles [0, nfull) go to the f workgroups of each query tile, the rest to the lw others:
            // the nfull near the even share that makes the slowest workgroup fastest (ties: larger)
            const int share = (int)((int64_t)f * pl.m_tiles * pl.n_tiles / num_cus);
            int nfull = 0, new_max = pl.n_tiles + 1;
            for (int cand = std::max(1, share - f); cand <= std::min(pl.n_tiles - 1, share + f); ++cand) {
                const int64_t rest = (int64_t)pl.m_tiles * (pl.n_tiles - cand);
                const int mx = (int)std::max<int64_t>((cand + f - 1) / f, (rest + lw - 1) / lw);
                if (mx <= new_max) {
                    new_max = mx;
                    nfull = cand;
                }
            }
            const int lo = pl.n_tiles - nfull;
            const int64_t total_lo = (int64_t)pl.m_tiles * lo;
            const int old_max = (pl.n_tiles + pl.n_splits - 1) / pl.n_splits;
            if (nfull > 0 && lo > 0 && lo <= total_lo / lw && new_max < old_max) {
                pl.bal_f = f;
                pl.bal_nfull = nfull;
                pl.bal_wgs = num_cus;
                pl.bal_lists = f + 2;
            }
        }
    }
    pl.sk_wgs = pl.sk_len = pl.sk_slots = 0;
    if (keys_out) plan_stream_k(pl, num_cus, d_pad);
    return pl;
}

// Stream-K for the keys-out variant when whole (query tile, cache tile) units fill the CUs badly
// (196 units on 256 CUs leave a quarter of the chip idle; 4 units nearly all of it) and the depth
// is long enough to be worth cutting.
void plan_stream_k(DistPlan &pl, int num_cus, int64_t d_pad)
{
    pl.sk_wgs = pl.sk_len = pl.sk_slots = 0;
    const int nk = (int)(d_pad / 32);   // k-steps per tile of the keys-out variant
    const int64_t tiles = (int64_t)pl.m_tiles * pl.n_tiles;
    const int64_t rounds = (tiles + num_cus - 1) / num_cus;
    const double fill = (double)tiles / ((double)rounds * num_cus);
    const int64_t total = tiles * nk;
    if (fill < 0.9 && rounds <= 4 && nk >= 64 && total >= 16 * (int64_t)num_cus) {
        pl.sk_wgs = num_cus;
        pl.sk_len = (int)((total + num_cus - 1) / num_cus);
        pl.sk_len += pl.sk_len & 1;   // the kernel takes k-steps in pairs (nk is even: d_pad is a multiple of 64)
        pl.sk_slots = (pl.sk_len - 1) / nk + 2;
    }
}

size_t dist_partial_bytes(const DistPlan &plan)
{
    return (size_t)plan.sk_wgs * plan.sk_slots * (size_t)plan.bm * kTileN * 4;
}

template <class C>
static hipError_t launch_variant(const DistPlan &plan, const DistArgs &a, hipStream_t s)
{
    DistKernelArgs k{};
    k.q_bf = a.q_bf;
    k.c_bf = a.c_bf;
    k.norm = a.norm;
    k.part = a.part;
    k.count = a.count;
    k.b = a.b;
    k.n = a.n;
    k.d_pad = a.d_pad;
    k.n_tiles = plan.n_tiles;
    k.n_splits = plan.n_splits;
    k.r = plan.r;
    k.alloc_splits = a.lists;
    k.max_splits = plan.max_splits;
    k.num_cus = plan.num_cus;
    const int grid = a.count ? plan.grid_units : plan.m_tiles * plan.n_splits;
    // the kernel takes k-steps (32 elements) in pairs
    if (a.d_pad <= 0 || a.d_pad % 64 != 0 || (plan.sk_wgs > 0 && (plan.sk_len & 1))) return hipErrorInvalidValue;
    if constexpr (!C::KEYS) {
        if (!a.part || a.lists < (a.count ? plan.alloc_splits : plan.n_splits)) return hipErrorInvalidValue;
    }
    k.keys = a.keys;
    k.bmin = a.bmin;
    k.projection = a.projection ? 1 : 0;
    k.relu = a.relu ? 1 : 0;
    k.n_pad = (int64_t)plan.n_tiles * kTileN;
    if constexpr (C::KEYS) {
        if (plan.sk_wgs > 0) {
            if (!a.partial || a.count) return hipErrorInvalidValue;
            k.partial = a.partial;
            k.sk_len = plan.sk_len;
            k.sk_slots = plan.sk_slots;
            hipLaunchKernelGGL((dist_topr_kernel<C>), dim3(plan.sk_wgs), dim3(C::THREADS), 0, s, k);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((keys_fixup_kernel<C>), dim3(plan.m_tiles * plan.n_tiles), dim3(C::THREADS), 0, s, k);
            return hipGetLastError();
        }
    }
    if constexpr (!C::KEYS) {
        if (a.balanced) {
            if (plan.bal_f <= 0 || a.count || a.lists < plan.bal_lists) return hipErrorInvalidValue;
            k.bal_f = plan.bal_f;
            k.bal_nfull = plan.bal_nfull;
            hipLaunchKernelGGL((dist_topr_kernel<C>), dim3(plan.bal_wgs), dim3(C::THREADS), 0, s, k);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((dist_topr_kernel<C>), dim3(grid), dim3(C::THREADS), 0, s, k);
    return hipGetLastError();
}

hipError_t launch_dist_topr(const DistPlan &plan, const DistArgs &a, hipStream_t s)
{
    if (plan.r < 1 || plan.r > kMaxRescore || a.d_pad % kPadD != 0) return hipErrorInvalidValue;
    if (plan.variant == 3 && (!a.keys || (!a.bmin && !a.projection))) return hipErrorInvalidValue;
    switch (plan.variant) {
    case 0: return launch_variant<DistCfg<256, 32, 16, 4, 2>>(plan, a, s);
    case 1: return launch_variant<DistCfg<256, 32, 32, 3>>(plan, a, s);
    case 2: return launch_variant<DistCfg<128, 32, 64, 4>>(plan, a, s);
    default:
        if (plan.sk_wgs > 0 && plan.m_tiles == 1) return launch_variant<DistCfg<256, 32, 0, 5, 4, true>>(plan, a, s);
        return launch_variant<DistCfg<256, 32, 0, 5>>(plan, a, s);
    }
}

}  // namespace fz
