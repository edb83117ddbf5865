// Distance pass for small batches (at most 16 queries): the bandwidth-bound path.
//
// With a handful of queries the look-up is a matrix-vector product: every cache entry is
// read once and used for a few dot products, so the kernel is built around streaming the
// cache from HBM exactly once with many bytes in flight, not around the matrix cores' rate.
// It computes the same ranking key as the batched kernel,
//     key(b, n) = |c_n|^2 - 2 * sum_i Q_bf[b,i] * C_bf[n,i]      (bf16 x bf16 -> fp32 MFMA),
// and keeps, per query and per range of cache tiles, the R entries with the smallest
// (key, index); the finishing kernel re-scores them exactly in fp32.
//
// Paper: Sec. 3 (k nearest neighbours of the layer output), Sec. 5 "Cache lookup
// performance" (look-up latency decides whether freezing pays off).
//
// Layout of the work: one workgroup per range of 256-entry cache tiles.  The prepared
// queries (a 32-row block for the matrix cores, rows past the batch zero) stay resident in
// LDS for the whole kernel.  The cache, stored in the tiled
// layout ([tile][k-block][row][32 elements]), is one contiguous stream per workgroup: it is
// copied verbatim into a ring of NS 16 KiB LDS stages with LDS-direct loads, NS-1 stages in
// flight, and the ring keeps running across tile boundaries so the epilogue of one tile
// overlaps the loads of the next.  Each of the 8 waves owns 32 of the tile's 256 entries:
// one 32x32x16 MFMA per 16 elements of k.  The tile's 256 squared norms travel the same way
// (one LDS-direct load per wave and tile), so no ordinary load ever drains the ring.  After
// the last k-block of a tile the keys go to a 16 x 256 slab in LDS; thread t (< batch) scans
// row t and inserts survivors into its top-R list.
#include "freeze_internal.h"

namespace fz {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void *lds_void_ptr;

namespace {

__device__ __forceinline__ void load16_global_to_lds(const void *g, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_byte_addr), "v"(g)
                 : "memory", "m0");
}
__device__ __forceinline__ void load4_global_to_lds(const void *g, uint32_t lds_byte_addr)
{
    // lane i lands at +4*i
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_byte_addr), "v"(g)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_global_loads_le() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

__device__ __forceinline__ uint32_t ordered_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t u)
{
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

constexpr int kMmaRows = 32;               // rows of the query block fed to the matrix cores
constexpr int kRows = kSkinnyRows;         // rows that can hold a query (the rest are zero)
constexpr int kStage = kTileN * kKB * 2;   // 16 KiB: one k-block of one cache tile
constexpr int kSlab = kRows * kTileN * 4;  // 16 KiB
constexpr int kTop = kMaxRescore * kRows * 8;   // 8 KiB
constexpr int kNormBuf = 2 * 8 * 256;      // 4 KiB: per tile parity and wave, 64 floats
static_assert(kRows <= 16, "slab rows are the first two row groups of the MFMA output");

template <int DMAX_, int NS_>
struct SkinnyCfg {
    static constexpr int DMAX = DMAX_, NS = NS_;
    static constexpr int A_BYTES = kMmaRows * DMAX * 2;
    static constexpr int LDS_BYTES = A_BYTES + kSlab + kTop + kNormBuf + NS * kStage;
    static_assert(LDS_BYTES <= 163840, "LDS budget");
    static_assert(NS >= 2 && NS <= 6, "stages");
};

struct SkinnyArgs {
    const uint16_t *q_bf;   // 32 x d_pad (rows >= b zero), tiled layout with 32-row tiles
    const uint16_t *c_bf;
    const float *norm;
    uint64_t *part;         // [b, n_splits, r]
    int b, n, d_pad, n_tiles, n_splits, r;
};

template <class C>
__global__ __launch_bounds__(512) void dist_skinny_kernel(SkinnyArgs p)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[C::LDS_BYTES];
    const bf16x8 *smem16 = reinterpret_cast<const bf16x8 *>(smem);
    float *slab = reinterpret_cast<float *>(smem + C::A_BYTES);                 // [16][256]
    uint64_t *top = reinterpret_cast<uint64_t *>(smem + C::A_BYTES + kSlab);    // [RMAX][16]
    constexpr int NORMS = C::A_BYTES + kSlab + kTop;                            // byte offset of the norm buffers
    const float *normbuf = reinterpret_cast<const float *>(smem + NORMS);       // [2][8 waves][64]
    constexpr int RING = NORMS + kNormBuf;                                      // byte offset of the stage ring

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sp = blockIdx.x;
    const int nt0 = (int)(((int64_t)sp * p.n_tiles) / p.n_splits);
    const int nt1 = (int)(((int64_t)(sp + 1) * p.n_tiles) / p.n_splits);
    const int r = p.r;
    const int kblocks = p.d_pad / kKB;                 // k-blocks per tile
    const int total = (nt1 - nt0) * kblocks;           // stages this workgroup streams
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_void_ptr)smem;

    uint64_t curmax = kSentinel;
    int maxpos = 0;
    float tau = __builtin_inff();
    if (tid < kRows) {
#pragma unroll
        for (int i = 0; i < kMaxRescore; ++i) top[i * kRows + tid] = kSentinel;
    }

    // the cache stream of this workgroup is contiguous: tiles nt0..nt1-1, each kblocks * 16 KiB
    const unsigned char *stream = reinterpret_cast<const unsigned char *>(p.c_bf) +
                                  (size_t)nt0 * kTileN * p.d_pad * 2 + w * 1024 + lane * 16;
    auto issue = [&](int slot, int gstep) {
        // 16 KiB = 16 wave-instructions of 1 KiB: two per wave
        const unsigned char *src = stream + (size_t)gstep * kStage;
        const uint32_t dst = smem_base + RING + slot * kStage + w * 1024;
        load16_global_to_lds(src, dst);
        load16_global_to_lds(src + 8192, dst + 8192);
    };
    constexpr int LPS = 2;   // loads per wave and stage
    // norms of this wave's 32 entries of tile `t` -> normbuf[t & 1][w][lane] (lanes 32..63 duplicate)
    auto issue_norms = [&](int t) {
        load4_global_to_lds(p.norm + (size_t)t * kTileN + w * 32 + (lane & 31),
                            smem_base + NORMS + ((t & 1) * 8 + w) * 256);
    };

    // queries -> LDS (linear copy of the prepared, tiled 32-row block), ordinary loads
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(p.q_bf);
        uint4 *dst = reinterpret_cast<uint4 *>(smem);
        for (int i = tid; i < kMmaRows * p.d_pad * 2 / 16; i += 512) dst[i] = src[i];
    }
    if (total > 0) issue_norms(nt0);
#pragma unroll
    for (int ps = 0; ps < C::NS - 1; ++ps)
        if (ps < total) issue(ps, ps);

    const int g = lane >> 5;
    const int rowA = lane & 31;
    const int rowB = w * 32 + (lane & 31);
    const int rdA = rowA * 4, pcxA = g ^ tiled_chunk_swizzle(rowA);
    const int rdB = rowB * 4, pcxB = g ^ tiled_chunk_swizzle(rowB);

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    int slot = 0, kb = 0, nt = nt0;
    for (int gs = 0; gs < total; ++gs) {
        // stage gs must have landed; up to NS-2 younger stages may stay in flight
        const int younger = total - 1 - gs;
        switch (younger < C::NS - 2 ? younger : C::NS - 2) {
        case 0: wait_global_loads_le<0>(); break;
        case 1: wait_global_loads_le<1 * LPS>(); break;
        case 2: wait_global_loads_le<2 * LPS>(); break;
        case 3: wait_global_loads_le<3 * LPS>(); break;
        default: wait_global_loads_le<4 * LPS>(); break;
        }
        __syncthreads();
        // The norms of the NEXT tile are requested at this tile's first step, before this step's
        // stage loads: they are older than every stage still in flight when they are read, and an
        // extra outstanding load only makes the counted waits above stricter.  (Their buffer was
        // last read at the end of the tile before this one: a barrier ago.)
        if (kb == 0 && nt + 1 < nt1) issue_norms(nt + 1);
        if (gs + C::NS - 1 < total) issue((slot + C::NS - 1) % C::NS, gs + C::NS - 1);

        const int baseA = kb * (kMmaRows * 4) + rdA;
        const int baseB = (RING + slot * kStage) / 16 + rdB;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const bf16x8 af = smem16[baseA + ((kk << 1) ^ pcxA)];
            const bf16x8 bfr = smem16[baseB + ((kk << 1) ^ pcxB)];
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc, 0, 0, 0);
        }
        slot = (slot + 1 == C::NS) ? 0 : slot + 1;
        if (++kb < kblocks) continue;

        // ---- tile finished: fold its 256 keys per query into the top-R lists ----
        kb = 0;
        const int n0 = nt * kTileN;
        ++nt;
        {
            // With fewer k-blocks than stages in flight the norm load may still be outstanding.
            if (kblocks < C::NS) wait_global_loads_le<0>();
            const int col = w * 32 + (lane & 31);
            const float nrm = normbuf[(((nt - 1) & 1) * 8 + w) * 64 + (lane & 31)];
#pragma unroll
            for (int e = 0; e < 8; ++e) {   // accumulator rows 0..15: the rows that can hold a query
                const int row = (e >> 2) * 8 + g * 4 + (e & 3);
                slab[row * kTileN + ((((col >> 2) ^ row) & 63) << 2) + (col & 3)] = __builtin_fmaf(-2.f, acc[e], nrm);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
        }
        __syncthreads();
        if (tid < p.b) {
            const int t = tid;
            const f32x4 *srow = reinterpret_cast<const f32x4 *>(slab + t * kTileN);
            const int lim = p.n - n0;   // columns < lim are real entries
#pragma unroll 1
            for (int m = 0; m < 4; ++m) {
                uint64_t mk = 0;
#pragma unroll 4
                for (int cgi = 0; cgi < 16; ++cgi) {
                    const int cg = m * 16 + cgi;
                    const f32x4 v = srow[(cg ^ t) & 63];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool pass = (v[e] <= tau) && (cg * 4 + e < lim);
                        mk |= (uint64_t)pass << (cgi * 4 + e);
                    }
                }
                while (mk) {
                    const int col = m * 64 + __builtin_ctzll(mk);
                    mk &= mk - 1;
                    const float key = slab[t * kTileN + ((((col >> 2) ^ t) & 63) << 2) + (col & 3)];
                    const uint64_t ent = ((uint64_t)ordered_bits(key) << 32) | (uint32_t)(n0 + col);
                    if (ent < curmax) {
                        top[maxpos * kRows + t] = ent;
                        curmax = 0;
                        for (int i = 0; i < r; ++i) {
                            const uint64_t v = top[i * kRows + t];
                            if (v >= curmax) { curmax = v; maxpos = i; }
                        }
                        tau = (curmax == kSentinel) ? __builtin_inff() : from_ordered_bits((uint32_t)(curmax >> 32));
                    }
                }
            }
        }
        // the next slab write happens after at least one more __syncthreads (next stage's)
    }
    if (tid < p.b) {
        uint64_t *dst = p.part + ((size_t)tid * p.n_splits + sp) * r;
        for (int i = 0; i < r; ++i) dst[i] = top[i * kRows + tid];
    }
}

}  // namespace

int plan_skinny_splits(int64_t n, int r, int num_cus)
{
    const int n_tiles = (int)((n + kTileN - 1) / kTileN);
    int s = num_cus < n_tiles ? num_cus : n_tiles;
    if (s > kMaxMergeEntries / r) s = kMaxMergeEntries / r;
    return s < 1 ? 1 : s;
}

hipError_t launch_dist_skinny(const DistArgs &a, int n_splits, int r, hipStream_t s)
{
    if (a.d_pad > kSkinnyMaxD || a.d_pad % kPadD != 0 || r < 1 || r > kMaxRescore || a.count != nullptr ||
        a.b > kSkinnyRows)
        return hipErrorInvalidValue;
    SkinnyArgs k{};
    k.q_bf = a.q_bf;
    k.c_bf = a.c_bf;
    k.norm = a.norm;
    k.part = a.part;
    k.b = a.b;
    k.n = a.n;
    k.d_pad = a.d_pad;
    k.n_tiles = (a.n + kTileN - 1) / kTileN;
    k.n_splits = n_splits;
    k.r = r;
    if (a.d_pad <= 512)
        hipLaunchKernelGGL((dist_skinny_kernel<SkinnyCfg<512, 6>>), dim3(n_splits), dim3(512), 0, s, k);
    else
        hipLaunchKernelGGL((dist_skinny_kernel<SkinnyCfg<1024, 4>>), dim3(n_splits), dim3(512), 0, s, k);
    return hipGetLastError();
}

}  // namespace fz
