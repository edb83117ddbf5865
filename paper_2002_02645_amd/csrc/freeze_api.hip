// C ABI of the library: argument checking, carving of the caller's storage / workspace
// buffers, and the launch sequences of the look-up and of the cascade.  Host code only;
// every step of the look-up itself runs in the HIP kernels.
#include "../../include/freeze.h"

#include <mutex>
#include <new>
#include <vector>

#include "freeze_internal.h"

using namespace fz;

struct freeze_ctx {
    std::vector<LayerCache> layers;
    int num_cus = 256;
    // stage timing (measurement aid): 4 events per recorded look-up
    int profile = 0;          // 0: off; 1: events at all four stage boundaries; 2: around the distance pass only;
                              // 3: as 2, for every eighth look-up
    unsigned profile_seen = 0;   // look-ups since profiling was enabled (mode 3 samples them)
    int profile_recorded = 0; // mode the recorded look-ups were taken in
    std::vector<hipEvent_t> events;
    int profiled_calls = 0;
    unsigned long long *stats = nullptr;   // device counters of the certificate's verdicts, or null
    int centring = 1;   // caches built from now on: 0 never centred, 1 when the mean dominates the spread, 2 always
};

// Scratch of freeze_lookup_static: the look-up's workspace for callers that cannot allocate.
// Every GPU the library runs on holds its own copy of this array until the process ends; host
// code never uses the array's name as an address, only what hipGetSymbolAddress returned for
// the device in question (static_scratch_ptr).
static __device__ __align__(256) unsigned char scratch[FREEZE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};   // per device: address of that device's copy of `scratch`

// Address of the current device's copy of `scratch`, resolved once per device with that device
// current.  Null (and *err set) when there is no usable device.
void *static_scratch_ptr(hipError_t *err)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *err = e;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            *err = e != hipSuccess ? e : hipErrorInvalidSymbol;
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *err = hipSuccess;
    return g_scratch_ptr[dev];
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// bump allocator over a caller-provided buffer
struct Carver {
    unsigned char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<unsigned char *>(p)) {}
    template <class T>
    T *take(size_t count)
    {
        T *p = reinterpret_cast<T *>(base + off);
        off += align_up(count * sizeof(T));
        return p;
    }
};

struct CacheLayout {
    int64_t n_pad, d_pad;
    size_t bytes;
};

bool cache_layout(int64_t n, int64_t d, int dtype, CacheLayout *out)
{
    if (n < 1 || n >= (int64_t)2147483647 - 512 || d < 1 || d > (1 << 24)) return false;
    if (dtype != FREEZE_F32 && dtype != FREEZE_BF16) return false;
    out->n_pad = round_up(n, kTileN);
    out->d_pad = round_up(d, kPadD);
    size_t bytes = align_up((size_t)out->n_pad * out->d_pad * 2) + align_up((size_t)out->n_pad * 4) +
                   align_up((size_t)n * 4);
    bytes += align_up((size_t)n * out->d_pad * (dtype == FREEZE_F32 ? 4 : 2));   // row-major copy for re-scoring
    bytes += align_up((size_t)out->d_pad * 4) + align_up((size_t)out->d_pad * 16);    // centring vector and its column statistics
    out->bytes = bytes;
    return true;
}

// (k = 1, the nearest centre of a k-means cache: eight candidates, the fewest the certificate takes its estimate from)
int default_rescore(int k) { return k == 1 ? 8 : (k <= 10 ? 16 : (k <= 24 ? 32 : 64)); }

// Validated parameters of one look-up on one layer.
struct LookupShape {
    int r;
    bool skinny;   // small-batch bandwidth-bound kernel instead of the tiled matrix-core kernel
    bool keys;     // tiled kernel writes every key; selection by the threshold / filter kernels
    bool cascade;  // sized for a look-up whose live count may sit on the device
    DistPlan plan;
    size_t ws_bytes;
};

// Candidate lists per query the distance pass writes (and their stride), by decomposition.
int lists_per_query(const DistPlan &pl, bool device_count)
{
    if (device_count) return pl.alloc_splits;
    return pl.bal_f > 0 ? pl.bal_lists : pl.n_splits;
}

bool lookup_shape(const freeze_ctx *ctx, const LayerCache &L, int64_t b, int k, int rescore_r, bool cascade,
                  LookupShape *out)
{
    if (b < 0 || b > (int64_t)1 << 30 || k < 1 || k > L.n) return false;
    if (k > FREEZE_MAX_K && !(k == L.n && k <= FREEZE_MAX_RESCORE)) return false;
    int r = rescore_r == 0 ? default_rescore(k) : rescore_r;
    if (rescore_r != 0 && (rescore_r < k || rescore_r > FREEZE_MAX_RESCORE)) return false;
    if (r < k) r = k;
    if ((int64_t)r > L.n) r = (int)L.n;
    out->r = r;
    out->cascade = cascade;
    // list and count of the queries the certificate flags, the exact scan's tickets and lists
    const size_t bb = (size_t)(b > 0 ? b : 1);
    const size_t scan_bytes = align_up(8) + 3 * align_up((bb > 2 * kSkinnyRows ? bb : 2 * kSkinnyRows) * 4) +
                              align_up(scan_scratch_entries(b, k, ctx->num_cus) * 8);
    out->skinny = !cascade && skinny_supported(b, L.n_pad, L.d_pad, r, ctx->num_cus);
    out->keys = false;
    if (out->skinny) {
        DistPlan pl{};
        pl.variant = -1;
        pl.bm = kSkinnyRows;   // the query block held by the streaming kernel
        pl.r = r;
        pl.m_tiles = 1;
        pl.n_tiles = (int)(L.n_pad / kTileN);
        pl.n_splits = plan_skinny_splits(L.n, ctx->num_cus);
        pl.b_pad = kSkinnyRows;
        out->plan = pl;
        out->ws_bytes = align_up((size_t)pl.b_pad * L.d_pad * 2) + skinny_workspace_bytes(L.n_pad, r, kAlign) + scan_bytes;
    } else {
        // One query tile and a long activation: materialising the keys (4 B per entry and query)
        // is cheap next to the cache stream (2 d B per entry), lets the tile be 256 queries wide for
        // any R, and keeps the selection out of the streaming kernel.  One query tile and a cache of
        // moderate size: every workgroup of the fused kernel gets a few tiles only and spends most of
        // its time filling its empty candidate lists key by key, so the keys go out here too
        // (measured cross-over: about 2^26 keys; 256 x 2,000: 129 -> 69 us, 200 x 50,000 x 512: 209 -> 80 us).
        out->keys = !cascade && b <= 256 && (b * 20 <= L.d_pad || b * L.n_pad <= ((int64_t)1 << 26)) &&
                    select_supported(L.n_pad, r);
        out->plan = plan_dist(b, L.n, r, ctx->num_cus, out->keys, L.d_pad);
        out->ws_bytes = align_up((size_t)out->plan.b_pad * L.d_pad * 2);
        if (out->keys)
            out->ws_bytes += select_workspace_bytes(out->plan.b_pad, L.n_pad, r, kAlign) +
                             align_up(dist_partial_bytes(out->plan));
        else
            out->ws_bytes += align_up((size_t)out->plan.b_pad * lists_per_query(out->plan, cascade) * r * 8);
        out->ws_bytes += scan_bytes;
    }
    return true;
}

const LayerCache *get_layer(const freeze_ctx *ctx, int layer, int *err)
{
    if (!ctx) {
        *err = FREEZE_EINVAL;
        return nullptr;
    }
    if (layer < 0 || layer >= (int)ctx->layers.size()) {
        *err = FREEZE_ELAYER;
        return nullptr;
    }
    if (!ctx->layers[layer].built || ctx->layers[layer].bias) {   // a projection is not a cache
        *err = FREEZE_ENOTBUILT;
        return nullptr;
    }
    *err = FREEZE_OK;
    return &ctx->layers[layer];
}

// Enqueue one look-up.  `sel` / `count` (device) restrict it to the live requests of a cascade.
// Records the next stage boundary of a profiled look-up (no-op when profiling is off).
struct StageMarks {
    freeze_ctx *ctx;
    hipStream_t s;
    int slot;   // event index of this call's first mark, or -1
    StageMarks(freeze_ctx *c, hipStream_t st) : ctx(c), s(st), slot(-1)
    {
        if (c && c->profile == 3 && (c->profile_seen++ % FREEZE_PROFILE_SAMPLE) != 0) return;
        if (c && c->profile && c->profiled_calls < FREEZE_PROFILE_MAX_CALLS) {
            slot = 4 * c->profiled_calls;
            while ((int)c->events.size() < slot + 4) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) {
                    slot = -1;
                    return;
                }
                c->events.push_back(e);
            }
        }
    }
    void mark(int i)
    {
        if (slot >= 0 && (ctx->profile == 1 || i == 1 || i == 2)) (void)hipEventRecord(ctx->events[slot + i], s);
    }
    void done()
    {
        if (slot >= 0) ++ctx->profiled_calls;
    }
};

// How the k neighbours become a label and a hit decision: the plurality count against an
// integer threshold, or the distance-weighted confidence of Sec. 3 against a float threshold.
struct HitRule {
    int weighted;
    int vote_threshold;
    float conf_threshold;
    float *out_conf;   // [b], weighted rule only
};

// `prepared`: the workspace still holds the bf16 copy of these very queries from an earlier call
// with the same shape (the k-means build looks the same points up round after round).
int enqueue_lookup(freeze_ctx *ctx, const LayerCache &L, const LookupShape &sh, const float *queries, const int32_t *sel,
                   const int32_t *count, int64_t b, int k, const HitRule &rule, int32_t *out_labels, uint8_t *out_hit,
                   int32_t *out_votes, int32_t *out_nbr_idx, float *out_nbr_dist, void *workspace, hipStream_t s,
                   bool prepared = false)
{
    Carver ws(workspace);
    uint16_t *q_bf = ws.take<uint16_t>((size_t)sh.plan.b_pad * L.d_pad);
    const size_t bb = (size_t)b > 2 * (size_t)kSkinnyRows ? (size_t)b : 2 * (size_t)kSkinnyRows;
    int32_t *flag_count = ws.take<int32_t>(2);
    int32_t *flag_list = ws.take<int32_t>(bb);
    int32_t *flag_list2 = ws.take<int32_t>(bb);
    int32_t *tickets = ws.take<int32_t>(bb);   // the exact scan's; the small-batch finishing kernel's follow at + kSkinnyRows
    uint64_t *scan_lists = ws.take<uint64_t>(scan_scratch_entries(b, k, ctx->num_cus));
    StageMarks marks(ctx, s);

    marks.mark(0);
    // (the small-batch streaming kernel converts its few queries itself); the first kernel of the
    // look-up also clears the flag count and the tickets
    if (!sh.skinny && prepared) {
        // only the flag counts start over (the exact scan leaves its tickets at zero)
        if (launch_fill_i32(flag_count, 0, 2, s) != hipSuccess) return FREEZE_EHIP;
    } else if (!sh.skinny && launch_query_prep(queries, sel, count, b, sh.plan.b_pad, sh.plan.bm, L.d, L.d_pad, q_bf,
                                               flag_count, tickets, L.mu, s) != hipSuccess) {
        return FREEZE_EHIP;
    }

    FinishArgs fa{};
    marks.mark(1);
    bool marked2 = false;
    const uint64_t *skinny_bmin = nullptr, *skinny_wgmin = nullptr;
    uint64_t *skinny_cand = nullptr, *skinny_samp = nullptr;
    if (sh.skinny) {
        SkinnyLaunch sl{};
        sl.queries = queries;
        sl.d = L.d;
        sl.c_bf = L.c_bf;
        sl.norm = L.norm;
        sl.mu = L.mu;
        sl.bmin = ws.take<uint64_t>((size_t)kSkinnyRows * (L.n_pad / 32));
        sl.wgmin = ws.take<uint64_t>((size_t)kSkinnyRows * (L.n_pad / kTileN));
        sl.flag_count = flag_count;
        sl.tickets = tickets;
        sl.b = (int)b;
        sl.n = (int)L.n;
        sl.d_pad = (int)L.d_pad;
        sl.r = sh.r;
        sl.n_splits = sh.plan.n_splits;
        sl.n_pad = L.n_pad;
        if (launch_skinny_stream(sl, s) != hipSuccess) return FREEZE_EHIP;
        marks.mark(2);
        marked2 = true;
        skinny_bmin = sl.bmin;
        skinny_wgmin = sl.wgmin;
        skinny_cand = ws.take<uint64_t>((size_t)kSkinnyRows * ((sh.r + 1) / 2) * 64);
        skinny_samp = ws.take<uint64_t>((size_t)kSkinnyRows * ((sh.r + 1) / 2) * 2);
    } else {
        DistArgs da{};
        da.q_bf = q_bf;
        da.c_bf = L.c_bf;
        da.norm = L.norm;
        da.count = count;
        da.b = (int)b;
        da.n = (int)L.n;
        da.d_pad = (int)L.d_pad;
        if (sh.keys) {
            const size_t rows = (size_t)sh.plan.b_pad;
            da.keys = ws.take<float>(rows * L.n_pad);
            da.bmin = ws.take<uint64_t>(rows * (L.n_pad / 32));
            int32_t *cand_count = ws.take<int32_t>(rows);
            uint64_t *cand = ws.take<uint64_t>(rows * 32 * sh.r);
            da.partial = sh.plan.sk_wgs > 0 ? ws.take<float>(dist_partial_bytes(sh.plan) / 4) : nullptr;
            if (launch_dist_topr(sh.plan, da, s) != hipSuccess) return FREEZE_EHIP;
            marks.mark(2);
            marked2 = true;
            if (launch_select(da.keys, da.bmin, L.n_pad, (int)L.n, (int)b, sh.r, cand_count, cand, s) != hipSuccess)
                return FREEZE_EHIP;
            fa.part = cand;
            fa.part_count = cand_count;
            fa.part_stride = 32 * sh.r;
            fa.n_splits = 1;
        } else {
            // the workspace was sized by sh.cascade; the balanced decomposition only goes with it off
            const int alloc = lists_per_query(sh.plan, sh.cascade);
            const bool balanced = !sh.cascade && sh.plan.bal_f > 0;
            uint64_t *part = ws.take<uint64_t>((size_t)sh.plan.b_pad * alloc * sh.r);
            da.part = part;
            da.balanced = balanced;
            da.lists = alloc;
            if (launch_dist_topr(sh.plan, da, s) != hipSuccess) return FREEZE_EHIP;
            fa.part = part;
            fa.n_splits = balanced ? alloc : sh.plan.n_splits;
            fa.alloc_splits = alloc;
            fa.bm = sh.plan.bm;
            fa.n_tiles = sh.plan.n_tiles;
            fa.num_cus = sh.plan.num_cus;
            fa.max_splits = sh.plan.max_splits;
        }
    }
    if (!marked2) marks.mark(2);

    fa.r = sh.r;
    fa.queries = queries;
    fa.sel = sel;
    fa.count = count;
    fa.b = (int)b;
    fa.n = (int)L.n;
    fa.d = L.d;
    fa.d_pad = L.d_pad;
    fa.c_rows = L.c_rows;
    fa.c_f32 = L.c_f32;
    fa.labels = L.labels;
    fa.k = k;
    fa.vote_threshold = rule.vote_threshold;
    fa.weighted = rule.weighted;
    fa.fraction = L.fraction;
    fa.conf_threshold = rule.conf_threshold;
    fa.out_conf = rule.out_conf;
    fa.out_labels = out_labels;
    fa.out_hit = out_hit;
    fa.out_votes = out_votes;
    fa.out_nbr_idx = out_nbr_idx;
    fa.out_nbr_dist = out_nbr_dist;
    fa.flag_count = flag_count;
    fa.flag_list = flag_list;
    fa.flag_list2 = flag_list2;
    fa.stats = ctx->stats;
    if (skinny_bmin) {
        if (launch_skinny_finish(fa, skinny_bmin, skinny_wgmin, L.n_pad / 32, sh.plan.n_splits,
                                 (int)(L.n_pad / kTileN), skinny_cand, skinny_samp, tickets + kSkinnyRows, s) != hipSuccess)
            return FREEZE_EHIP;
    } else if (launch_finish(fa, ctx->num_cus, s) != hipSuccess) {
        return FREEZE_EHIP;
    }
    // the queries whose result the certificate did not confirm (usually none) are redone exactly
    if (launch_exact_scan(fa, tickets, scan_lists, ctx->num_cus, s) != hipSuccess) return FREEZE_EHIP;
    marks.mark(3);
    marks.done();
    return FREEZE_OK;
}

struct CascadeLayout {
    size_t lookup_ws;   // largest per-layer look-up workspace
    size_t bytes;
};

bool cascade_layout(const freeze_ctx *ctx, int num_layers, const int *layers, int64_t b, int k, int rescore_r,
                    CascadeLayout *out, int *err)
{
    if (!ctx || !layers || num_layers < 1 || num_layers > 1024) {
        *err = FREEZE_EINVAL;
        return false;
    }
    size_t mx = 0;
    for (int l = 0; l < num_layers; ++l) {
        const LayerCache *L = get_layer(ctx, layers[l], err);
        if (!L) return false;
        // a layer is looked up either with the live count on the device (later layers of a cascade)
        // or with all b requests (its first layer; every layer while thresholds are calibrated)
        LookupShape sh, sh_all;
        if (!lookup_shape(ctx, *L, b, k, rescore_r, true, &sh) || !lookup_shape(ctx, *L, b, k, rescore_r, false, &sh_all)) {
            *err = FREEZE_EINVAL;
            return false;
        }
        if (sh.ws_bytes > mx) mx = sh.ws_bytes;
        if (sh_all.ws_bytes > mx) mx = sh_all.ws_bytes;
    }
    out->lookup_ws = mx;
    const size_t bb = (size_t)(b > 0 ? b : 1);
    // per-layer outputs in compact order + two miss lists + two counters
    out->bytes = mx + 3 * align_up(bb * 4) + align_up(bb) + 2 * align_up(bb * k * 4) + 2 * align_up(bb * 4) +
                 2 * align_up(4);
    *err = FREEZE_OK;
    return true;
}

// Which confidence applies on a layer: the distance-weighted heuristic of Sec. 3 on a k-NN cache,
// majority share over distance on a k-means cache (Sec. 4), which is defined for k = 1 only.
int confidence_rule_for(const freeze_ctx *ctx, int layer, int k, int *kind)
{
    int err;
    const LayerCache *L = get_layer(ctx, layer, &err);
    if (!L) return err;
    *kind = L->fraction ? 2 : 1;
    if (L->fraction && k != 1) return FREEZE_EINVAL;
    return FREEZE_OK;
}

int lookup_checked(freeze_ctx *ctx, int layer, const float *queries, int64_t b, int k, const HitRule &rule,
                   int rescore_r, int32_t *out_labels, uint8_t *out_hit, int32_t *out_votes, int32_t *out_nbr_idx,
                   float *out_nbr_dist, void *workspace, size_t workspace_bytes, void *stream)
{
    int err;
    const LayerCache *L = get_layer(ctx, layer, &err);
    if (!L) return err;
    LookupShape sh;
    if (!lookup_shape(ctx, *L, b, k, rescore_r, false, &sh)) return FREEZE_EINVAL;
    if (b == 0) return FREEZE_OK;   // nothing to look up: data pointers may be null
    if (!queries || !out_labels || !out_hit || !out_votes || !out_nbr_idx || !out_nbr_dist || !workspace)
        return FREEZE_EINVAL;
    if ((reinterpret_cast<uintptr_t>(queries) % 16) != 0) return FREEZE_EINVAL;
    if (workspace_bytes < sh.ws_bytes || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return FREEZE_EWORKSPACE;
    return enqueue_lookup(ctx, *L, sh, queries, nullptr, nullptr, b, k, rule, out_labels, out_hit, out_votes,
                          out_nbr_idx, out_nbr_dist, workspace, static_cast<hipStream_t>(stream));
}

// The cascade of Pseudocode 1 (FreezeInference) under either hit rule; `rules` has one entry per
// position in `layers` (out_conf is filled in here).
int cascade_checked(freeze_ctx *ctx, int num_layers, const int *layers, const float *const *queries_per_layer,
                    int64_t b, int k, const std::vector<HitRule> &rules, int rescore_r, int32_t *out_labels,
                    int32_t *out_exit_layer, int64_t *out_hits_per_layer, void *workspace, size_t workspace_bytes,
                    void *stream)
{
    CascadeLayout cl;
    int err;
    if (!cascade_layout(ctx, num_layers, layers, b, k, rescore_r, &cl, &err)) return err;
    if (!queries_per_layer || !out_hits_per_layer || !workspace) return FREEZE_EINVAL;
    if (b > 0 && (!out_labels || !out_exit_layer)) return FREEZE_EINVAL;
    for (int l = 0; l < num_layers; ++l) {
        if (b > 0 && (!queries_per_layer[l] || (reinterpret_cast<uintptr_t>(queries_per_layer[l]) % 16) != 0))
            return FREEZE_EINVAL;
    }
    if (workspace_bytes < cl.bytes || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return FREEZE_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    Carver ws(workspace);
    unsigned char *lookup_ws = ws.take<unsigned char>(cl.lookup_ws);
    const size_t bb = (size_t)(b > 0 ? b : 1);
    int32_t *t_labels = ws.take<int32_t>(bb);
    int32_t *t_votes = ws.take<int32_t>(bb);
    float *t_conf = ws.take<float>(bb);
    uint8_t *t_hit = ws.take<uint8_t>(bb);
    int32_t *t_idx = ws.take<int32_t>(bb * k);
    float *t_dist = ws.take<float>(bb * k);
    int32_t *sel_buf[2] = {ws.take<int32_t>(bb), ws.take<int32_t>(bb)};
    int32_t *cnt_buf[2] = {ws.take<int32_t>(1), ws.take<int32_t>(1)};

    if (b == 0) {
        // nothing to look up: every layer froze zero requests
        for (int l = 0; l < num_layers; ++l)
            if (launch_compact(t_hit, nullptr, nullptr, 0, sel_buf[0], cnt_buf[0], out_hits_per_layer + l, s) !=
                hipSuccess)
                return FREEZE_EHIP;
        return FREEZE_OK;
    }
    if (launch_cascade_init(out_labels, out_exit_layer, b, s) != hipSuccess) return FREEZE_EHIP;

    const int32_t *sel = nullptr;     // layer 0: every request, identity order
    const int32_t *count = nullptr;
    for (int l = 0; l < num_layers; ++l) {
        const LayerCache &L = ctx->layers[layers[l]];
        // Every request enters the first layer: its look-up is planned like a single-layer one, with
        // the count known on the host (any route, any decomposition); the later layers are sized for
        // b and read the live count on the device.
        LookupShape sh;
        lookup_shape(ctx, L, b, k, rescore_r, l != 0, &sh);
        HitRule rule = rules[(size_t)l];
        rule.out_conf = t_conf;
        int rc = enqueue_lookup(ctx, L, sh, queries_per_layer[l], sel, count, b, k, rule, t_labels, t_hit, t_votes,
                                t_idx, t_dist, lookup_ws, s);
        if (rc != FREEZE_OK) return rc;
        if (launch_cascade_scatter(t_labels, t_hit, sel, count, b, l, out_labels, out_exit_layer, s) != hipSuccess)
            return FREEZE_EHIP;
        int32_t *sel_next = sel_buf[l & 1];
        int32_t *cnt_next = cnt_buf[l & 1];
        if (launch_compact(t_hit, sel, count, b, sel_next, cnt_next, out_hits_per_layer + l, s) != hipSuccess)
            return FREEZE_EHIP;
        sel = sel_next;
        count = cnt_next;
    }
    return FREEZE_OK;
}

struct KmeansLayout {
    size_t lookup_ws;
    size_t bytes;
};
// workspace: two centre buffers, dummy labels, the look-up's outputs for n points and its workspace
bool kmeans_layout(const freeze_ctx *ctx, int64_t n, int64_t d, int64_t kc, KmeansLayout *out)
{
    CacheLayout cl;
    if (!ctx || n < 1 || n > (int64_t)1 << 30 || kc < 1 || kc > n || !cache_layout(kc, d, FREEZE_F32, &cl)) return false;
    LayerCache tmp;   // shape of the centres as a cache
    tmp.n = kc;
    tmp.d = d;
    tmp.n_pad = cl.n_pad;
    tmp.d_pad = cl.d_pad;
    LookupShape sh;
    if (!lookup_shape(ctx, tmp, n, 1, 0, false, &sh)) return false;
    out->lookup_ws = sh.ws_bytes;
    out->bytes = sh.ws_bytes + 2 * align_up((size_t)kc * d * 4) + align_up((size_t)kc * 4) + 3 * align_up((size_t)n * 4) +
                 align_up((size_t)n) + 2 * align_up((size_t)n * 4) +
                 align_up((size_t)kc * 4) + align_up((size_t)(kc + 1) * 4) + align_up((size_t)n * 4);   // grouping by centre
    return true;
}

const LayerCache *get_projection(const freeze_ctx *ctx, int slot, int *err)
{
    if (!ctx) {
        *err = FREEZE_EINVAL;
        return nullptr;
    }
    if (slot < 0 || slot >= (int)ctx->layers.size()) {
        *err = FREEZE_ELAYER;
        return nullptr;
    }
    if (!ctx->layers[slot].built || !ctx->layers[slot].bias) {
        *err = FREEZE_ENOTBUILT;
        return nullptr;
    }
    *err = FREEZE_OK;
    return &ctx->layers[slot];
}
// one workgroup per (tile of 256 inputs, tile of 256 outputs), whole depth
DistPlan projection_plan(const freeze_ctx *ctx, const LayerCache &P, int64_t b)
{
    DistPlan pl{};
    pl.variant = 3;
    pl.bm = 256;
    pl.r = 1;
    pl.m_tiles = (int)((b + 255) / 256);
    if (pl.m_tiles < 1) pl.m_tiles = 1;
    pl.n_tiles = (int)(P.n_pad / kTileN);
    pl.n_splits = pl.alloc_splits = pl.n_tiles;
    pl.max_splits = pl.n_tiles;
    pl.grid_units = pl.m_tiles * pl.n_tiles;
    pl.num_cus = ctx->num_cus;
    pl.b_pad = (int64_t)pl.m_tiles * 256;
    plan_stream_k(pl, ctx->num_cus, P.d_pad);
    return pl;
}

}  // namespace

extern "C" {

int freeze_create(freeze_ctx **out, int num_layers)
{
    if (!out || num_layers < 1 || num_layers > 65536) return FREEZE_EINVAL;
    freeze_ctx *c = new (std::nothrow) freeze_ctx;
    if (!c) return FREEZE_EINVAL;
    c->layers.resize((size_t)num_layers);
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        c->num_cus = prop.multiProcessorCount;
    else
        (void)hipGetLastError();   // no device: keep the MI355X default; launches will report the error
    // set-up of freeze_lookup_static for this device (it resolves the address itself when a context
    // is later used on another device, and reports the error there if this attempt failed)
    hipError_t scratch_err;
    (void)static_scratch_ptr(&scratch_err);
    *out = c;
    return FREEZE_OK;
}

int freeze_destroy(freeze_ctx *ctx)
{
    if (!ctx) return FREEZE_EINVAL;
    for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
    delete ctx;
    return FREEZE_OK;
}

size_t freeze_cache_storage_bytes(int64_t n, int64_t d, int entries_dtype)
{
    CacheLayout cl;
    return cache_layout(n, d, entries_dtype, &cl) ? cl.bytes : 0;
}

}  // extern "C"

namespace {
// allow_centre: false for what is not a cache of its own (the rows of a projection: a product is not
// invariant under a shift) and for the k-means rounds (the prepared copy of the points is reused
// across rounds, while the centres, and with them their mean, move)
int cache_build_impl(freeze_ctx *ctx, int layer, const void *entries, int entries_dtype, int64_t n, int64_t d,
                     const int32_t *labels, int32_t num_classes, void *storage, size_t storage_bytes, void *stream,
                     bool allow_centre)
{
    if (!ctx || !entries || !labels || !storage || num_classes < 1) return FREEZE_EINVAL;
    if (layer < 0 || layer >= (int)ctx->layers.size()) return FREEZE_ELAYER;
    CacheLayout cl;
    if (!cache_layout(n, d, entries_dtype, &cl)) return FREEZE_EINVAL;
    if (storage_bytes < cl.bytes || (reinterpret_cast<uintptr_t>(storage) % kAlign) != 0) return FREEZE_EWORKSPACE;

    Carver st(storage);
    uint16_t *c_bf = st.take<uint16_t>((size_t)cl.n_pad * cl.d_pad);
    float *norm = st.take<float>((size_t)cl.n_pad);
    int32_t *lab = st.take<int32_t>((size_t)n);
    float *c_f32 = entries_dtype == FREEZE_F32 ? st.take<float>((size_t)n * cl.d_pad) : nullptr;
    uint16_t *c_rows = entries_dtype == FREEZE_BF16 ? st.take<uint16_t>((size_t)n * cl.d_pad) : nullptr;
    float *mu = st.take<float>((size_t)cl.d_pad);
    double *col_stats = st.take<double>(2 * (size_t)cl.d_pad);
    const bool centre = allow_centre && ctx->centring != 0;

    LayerCache &L = ctx->layers[layer];
    L.built = false;
    if (launch_cache_build(entries, entries_dtype, n, d, cl.n_pad, cl.d_pad, c_bf, norm, c_f32, c_rows, labels, lab,
                           centre ? mu : nullptr, col_stats, ctx->centring, static_cast<hipStream_t>(stream)) != hipSuccess)
        return FREEZE_EHIP;
    L.n = n;
    L.d = d;
    L.n_pad = cl.n_pad;
    L.d_pad = cl.d_pad;
    L.num_classes = num_classes;
    L.entries_dtype = entries_dtype;
    L.c_bf = c_bf;
    L.norm = norm;
    L.labels = lab;
    L.c_f32 = c_f32;
    L.c_rows = c_rows;
    L.fraction = nullptr;
    L.bias = nullptr;
    L.mu = centre ? mu : nullptr;
    L.built = true;
    return FREEZE_OK;
}
}  // namespace

extern "C" {

int freeze_cache_build(freeze_ctx *ctx, int layer, const void *entries, int entries_dtype, int64_t n, int64_t d,
                       const int32_t *labels, int32_t num_classes, void *storage, size_t storage_bytes, void *stream)
{
    return cache_build_impl(ctx, layer, entries, entries_dtype, n, d, labels, num_classes, storage, storage_bytes, stream,
                            true);
}

int freeze_set_centring(freeze_ctx *ctx, int mode)
{
    if (!ctx || mode < 0 || mode > 2) return FREEZE_EINVAL;
    ctx->centring = mode;
    return FREEZE_OK;
}

size_t freeze_lookup_workspace_bytes(const freeze_ctx *ctx, int layer, int64_t b, int k, int rescore_r)
{
    int err;
    const LayerCache *L = get_layer(ctx, layer, &err);
    LookupShape sh;
    if (!L || !lookup_shape(ctx, *L, b, k, rescore_r, false, &sh)) return 0;
    return sh.ws_bytes;
}

int freeze_lookup(freeze_ctx *ctx, int layer, const float *queries, int64_t b, int k, int vote_threshold,
                  int rescore_r, int32_t *out_labels, uint8_t *out_hit, int32_t *out_votes, int32_t *out_nbr_idx,
                  float *out_nbr_dist, void *workspace, size_t workspace_bytes, void *stream)
{
    if (vote_threshold < 1 || vote_threshold > k) return FREEZE_EINVAL;
    const HitRule rule{0, vote_threshold, 0.f, nullptr};
    return lookup_checked(ctx, layer, queries, b, k, rule, rescore_r, out_labels, out_hit, out_votes, out_nbr_idx,
                          out_nbr_dist, workspace, workspace_bytes, stream);
}

int freeze_lookup_static(freeze_ctx *ctx, int layer, const float *queries, int64_t b, int k, int vote_threshold,
                         int rescore_r, int32_t *out_labels, uint8_t *out_hit, int32_t *out_votes, int32_t *out_nbr_idx,
                         float *out_nbr_dist, void *stream)
{
    if (vote_threshold < 1 || vote_threshold > k) return FREEZE_EINVAL;
    int err;
    const LayerCache *L = get_layer(ctx, layer, &err);
    if (!L) return err;
    LookupShape sh;
    if (!lookup_shape(ctx, *L, b, k, rescore_r, false, &sh)) return FREEZE_EINVAL;
    if (sh.ws_bytes > (size_t)FREEZE_STATIC_SCRATCH_BYTES) return FREEZE_ESCRATCH;
    if (b == 0) return FREEZE_OK;
    hipError_t herr;
    void *ws = static_scratch_ptr(&herr);
    if (!ws) return FREEZE_EHIP;
    const HitRule rule{0, vote_threshold, 0.f, nullptr};
    return lookup_checked(ctx, layer, queries, b, k, rule, rescore_r, out_labels, out_hit, out_votes, out_nbr_idx,
                          out_nbr_dist, ws, (size_t)FREEZE_STATIC_SCRATCH_BYTES, stream);
}

int freeze_lookup_confidence(freeze_ctx *ctx, int layer, const float *queries, int64_t b, int k, float conf_threshold,
                             int rescore_r, int32_t *out_labels, uint8_t *out_hit, float *out_conf,
                             int32_t *out_votes, int32_t *out_nbr_idx, float *out_nbr_dist, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    if (!(conf_threshold >= 0.f)) return FREEZE_EINVAL;   // also rejects NaN
    if (b > 0 && !out_conf) return FREEZE_EINVAL;
    int kind = 1;
    if (int rc = confidence_rule_for(ctx, layer, k, &kind)) return rc;
    const HitRule rule{kind, 1, conf_threshold, out_conf};
    return lookup_checked(ctx, layer, queries, b, k, rule, rescore_r, out_labels, out_hit, out_votes, out_nbr_idx,
                          out_nbr_dist, workspace, workspace_bytes, stream);
}

size_t freeze_cascade_workspace_bytes(const freeze_ctx *ctx, int num_layers, const int *layers, int64_t b, int k,
                                      int rescore_r)
{
    CascadeLayout cl;
    int err;
    return cascade_layout(ctx, num_layers, layers, b, k, rescore_r, &cl, &err) ? cl.bytes : 0;
}

int freeze_lookup_cascade(freeze_ctx *ctx, int num_layers, const int *layers, const float *const *queries_per_layer,
                          int64_t b, int k, const int *vote_thresholds, int rescore_r, int32_t *out_labels,
                          int32_t *out_exit_layer, int64_t *out_hits_per_layer, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    if (!vote_thresholds || num_layers < 1 || num_layers > 1024) return FREEZE_EINVAL;
    std::vector<HitRule> rules((size_t)num_layers);
    for (int l = 0; l < num_layers; ++l) {
        if (vote_thresholds[l] < 1 || vote_thresholds[l] > k) return FREEZE_EINVAL;
        rules[(size_t)l] = HitRule{0, vote_thresholds[l], 0.f, nullptr};
    }
    return cascade_checked(ctx, num_layers, layers, queries_per_layer, b, k, rules, rescore_r, out_labels,
                           out_exit_layer, out_hits_per_layer, workspace, workspace_bytes, stream);
}

int freeze_lookup_cascade_confidence(freeze_ctx *ctx, int num_layers, const int *layers,
                                     const float *const *queries_per_layer, int64_t b, int k,
                                     const float *conf_thresholds, int rescore_r, int32_t *out_labels,
                                     int32_t *out_exit_layer, int64_t *out_hits_per_layer, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    if (!conf_thresholds || num_layers < 1 || num_layers > 1024) return FREEZE_EINVAL;
    std::vector<HitRule> rules((size_t)num_layers);
    for (int l = 0; l < num_layers; ++l) {
        if (!(conf_thresholds[l] >= 0.f) || !layers) return FREEZE_EINVAL;
        int kind = 1;
        if (int rc = confidence_rule_for(ctx, layers[l], k, &kind)) return rc;
        rules[(size_t)l] = HitRule{kind, 1, conf_thresholds[l], nullptr};
    }
    return cascade_checked(ctx, num_layers, layers, queries_per_layer, b, k, rules, rescore_r, out_labels,
                           out_exit_layer, out_hits_per_layer, workspace, workspace_bytes, stream);
}

int freeze_compute_thresholds(freeze_ctx *ctx, int num_layers, const int *layers,
                              const float *const *queries_per_layer, int64_t b, int k, int rescore_r,
                              const int32_t *model_labels, float *out_thresholds, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    CascadeLayout cl;
    int err;
    if (!cascade_layout(ctx, num_layers, layers, b, k, rescore_r, &cl, &err)) return err;
    if (!queries_per_layer || !out_thresholds || !workspace) return FREEZE_EINVAL;
    if (b > 0 && !model_labels) return FREEZE_EINVAL;
    for (int l = 0; l < num_layers; ++l)
        if (b > 0 && (!queries_per_layer[l] || (reinterpret_cast<uintptr_t>(queries_per_layer[l]) % 16) != 0))
            return FREEZE_EINVAL;
    if (workspace_bytes < cl.bytes || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return FREEZE_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    Carver ws(workspace);
    unsigned char *lookup_ws = ws.take<unsigned char>(cl.lookup_ws);
    const size_t bb = (size_t)(b > 0 ? b : 1);
    int32_t *t_labels = ws.take<int32_t>(bb);
    int32_t *t_votes = ws.take<int32_t>(bb);
    float *t_conf = ws.take<float>(bb);
    uint8_t *t_hit = ws.take<uint8_t>(bb);
    int32_t *t_idx = ws.take<int32_t>(bb * k);
    float *t_dist = ws.take<float>(bb * k);

    if (launch_threshold_init(out_thresholds, num_layers, s) != hipSuccess) return FREEZE_EHIP;
    if (b == 0) return FREEZE_OK;
    // every validation item is looked up at every layer (no early exit while calibrating)
    for (int l = 0; l < num_layers; ++l) {
        const LayerCache &L = ctx->layers[layers[l]];
        LookupShape sh;
        lookup_shape(ctx, L, b, k, rescore_r, false, &sh);
        int kind = 1;
        if (int rck = confidence_rule_for(ctx, layers[l], k, &kind)) return rck;
        const HitRule rule{kind, 1, 0.f, t_conf};
        int rc = enqueue_lookup(ctx, L, sh, queries_per_layer[l], nullptr, nullptr, b, k, rule, t_labels, t_hit, t_votes,
                                t_idx, t_dist, lookup_ws, s);
        if (rc != FREEZE_OK) return rc;
        if (launch_threshold_max(t_labels, t_conf, model_labels, b, out_thresholds + l, s) != hipSuccess)
            return FREEZE_EHIP;
    }
    return FREEZE_OK;
}

size_t freeze_kmeans_storage_bytes(int64_t num_centers, int64_t d)
{
    CacheLayout cl;
    if (!cache_layout(num_centers, d, FREEZE_F32, &cl)) return 0;
    return cl.bytes + align_up((size_t)num_centers * 4);
}

size_t freeze_kmeans_workspace_bytes(const freeze_ctx *ctx, int64_t n, int64_t d, int64_t num_centers)
{
    KmeansLayout kl;
    return kmeans_layout(ctx, n, d, num_centers, &kl) ? kl.bytes : 0;
}

int freeze_kmeans_build(freeze_ctx *ctx, int layer, const float *points, int64_t n, int64_t d, const int32_t *labels,
                        int32_t num_classes, const float *init_centers, int64_t num_centers, int iters, void *storage,
                        size_t storage_bytes, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!ctx || !points || !labels || !init_centers || !storage || !workspace || iters < 0 || iters > 1000 ||
        num_classes < 1 || num_classes > 8192)
        return FREEZE_EINVAL;
    if (layer < 0 || layer >= (int)ctx->layers.size()) return FREEZE_ELAYER;
    KmeansLayout kl;
    if (!kmeans_layout(ctx, n, d, num_centers, &kl)) return FREEZE_EINVAL;
    if ((reinterpret_cast<uintptr_t>(points) % 16) != 0) return FREEZE_EINVAL;
    const size_t st_bytes = freeze_kmeans_storage_bytes(num_centers, d);
    if (storage_bytes < st_bytes || (reinterpret_cast<uintptr_t>(storage) % kAlign) != 0) return FREEZE_EWORKSPACE;
    if (workspace_bytes < kl.bytes || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0) return FREEZE_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t kc = num_centers;

    Carver ws(workspace);
    unsigned char *lookup_ws = ws.take<unsigned char>(kl.lookup_ws);
    float *cen[2] = {ws.take<float>((size_t)kc * d), ws.take<float>((size_t)kc * d)};
    int32_t *zero_labels = ws.take<int32_t>((size_t)kc);
    int32_t *t_labels = ws.take<int32_t>((size_t)n);
    int32_t *t_votes = ws.take<int32_t>((size_t)n);
    int32_t *assign = ws.take<int32_t>((size_t)n);
    uint8_t *t_hit = ws.take<uint8_t>((size_t)n);
    float *t_dist = ws.take<float>((size_t)n);
    float *t_conf = ws.take<float>((size_t)n);
    (void)t_conf;
    int32_t *grp_sizes = ws.take<int32_t>((size_t)kc);
    int32_t *grp_offsets = ws.take<int32_t>((size_t)kc + 1);
    int32_t *grp_members = ws.take<int32_t>((size_t)n);

    CacheLayout cl;
    cache_layout(kc, d, FREEZE_F32, &cl);
    float *fraction = reinterpret_cast<float *>(static_cast<unsigned char *>(storage) + cl.bytes);

    if (launch_copy_rows_f32(init_centers, d, cen[0], kc, d, s) != hipSuccess) return FREEZE_EHIP;
    if (launch_fill_i32(zero_labels, 0, kc, s) != hipSuccess) return FREEZE_EHIP;
    // rounds of (centres -> cache, every point looked up with k = 1, centres <- means); a last
    // assignment to the final centres gives the majority labels and their shares
    const HitRule rule{0, 1, 0.f, nullptr};
    for (int it = 0; it <= iters; ++it) {
        const float *cur = cen[it & 1];
        int rc = cache_build_impl(ctx, layer, cur, FREEZE_F32, kc, d, zero_labels, num_classes, storage, cl.bytes, stream, false);
        if (rc != FREEZE_OK) return rc;
        const LayerCache &L = ctx->layers[layer];
        LookupShape sh;
        if (!lookup_shape(ctx, L, n, 1, 0, false, &sh)) return FREEZE_EINVAL;
        // the points do not change from round to round: their bf16 copy is made once (the shape of
        // the look-up, and with it the layout of its workspace, is the same in every round)
        rc = enqueue_lookup(ctx, L, sh, points, nullptr, nullptr, n, 1, rule, t_labels, t_hit, t_votes, assign, t_dist,
                            lookup_ws, s, it > 0);
        if (rc != FREEZE_OK) return rc;
        if (it < iters &&
            launch_kmeans_update(points, assign, n, d, kc, cur, cen[(it + 1) & 1], grp_sizes, grp_offsets, grp_members, s) !=
                hipSuccess)
            return FREEZE_EHIP;
    }
    LayerCache &L = ctx->layers[layer];
    // the cache's label array becomes the majority labels, the shares go behind the cache
    if (launch_kmeans_majority(assign, labels, n, num_classes, kc, const_cast<int32_t *>(L.labels), fraction, nullptr, s) !=
        hipSuccess)
        return FREEZE_EHIP;
    L.fraction = fraction;
    return FREEZE_OK;
}

int freeze_kmeans_read(freeze_ctx *ctx, int layer, float *out_centers, int32_t *out_majority, float *out_fraction,
                       void *stream)
{
    int err;
    const LayerCache *L = get_layer(ctx, layer, &err);
    if (!L) return err;
    if (!L->fraction || !L->c_f32 || !out_centers || !out_majority || !out_fraction) return FREEZE_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (launch_copy_rows_f32(L->c_f32, L->d_pad, out_centers, L->n, L->d, s) != hipSuccess) return FREEZE_EHIP;
    if (launch_copy_rows_f32(L->fraction, 1, out_fraction, L->n, 1, s) != hipSuccess) return FREEZE_EHIP;
    if (launch_copy_i32(L->labels, out_majority, L->n, s) != hipSuccess) return FREEZE_EHIP;
    return FREEZE_OK;
}

size_t freeze_projection_storage_bytes(int64_t m, int64_t d, int weights_dtype)
{
    CacheLayout cl;
    if (!cache_layout(m, d, weights_dtype, &cl)) return 0;
    return cl.bytes + align_up((size_t)cl.n_pad * 4);
}

int freeze_projection_build(freeze_ctx *ctx, int slot, const void *weights, int weights_dtype, int64_t m, int64_t d,
                            const float *bias, void *storage, size_t storage_bytes, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    if (!ctx || !weights || !bias || !storage || !workspace) return FREEZE_EINVAL;
    if (slot < 0 || slot >= (int)ctx->layers.size()) return FREEZE_ELAYER;
    CacheLayout cl;
    if (!cache_layout(m, d, weights_dtype, &cl)) return FREEZE_EINVAL;
    if (storage_bytes < cl.bytes + align_up((size_t)cl.n_pad * 4) || (reinterpret_cast<uintptr_t>(storage) % kAlign) != 0)
        return FREEZE_EWORKSPACE;
    if (workspace_bytes < align_up((size_t)m * 4) || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return FREEZE_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the rows of W go through the cache ingest (bf16, tiled); its labels are not used
    int32_t *dummy_labels = static_cast<int32_t *>(workspace);
    if (launch_fill_i32(dummy_labels, 0, m, s) != hipSuccess) return FREEZE_EHIP;
    int rc = cache_build_impl(ctx, slot, weights, weights_dtype, m, d, dummy_labels, 1, storage, cl.bytes, stream, false);
    if (rc != FREEZE_OK) return rc;
    float *bias_pad = reinterpret_cast<float *>(static_cast<unsigned char *>(storage) + cl.bytes);
    if (launch_fill_i32(reinterpret_cast<int32_t *>(bias_pad), 0, cl.n_pad, s) != hipSuccess) return FREEZE_EHIP;
    if (launch_copy_rows_f32(bias, 1, bias_pad, m, 1, s) != hipSuccess) return FREEZE_EHIP;
    ctx->layers[slot].bias = bias_pad;
    return FREEZE_OK;
}

size_t freeze_project_workspace_bytes(const freeze_ctx *ctx, int slot, int64_t b)
{
    int err;
    const LayerCache *P = get_projection(ctx, slot, &err);
    if (!P || b < 0 || b > (int64_t)1 << 30) return 0;
    const int64_t b_pad = (b + 255) / 256 * 256 + (b == 0 ? 256 : 0);
    const DistPlan pl = projection_plan(ctx, *P, b);
    return align_up((size_t)b_pad * P->d_pad * 2) + align_up((size_t)(b > 0 ? b : 1) * P->n_pad * 4) +
           align_up(dist_partial_bytes(pl));
}

int freeze_project(freeze_ctx *ctx, int slot, const float *x, int64_t b, int relu, float *out, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    int err;
    const LayerCache *P = get_projection(ctx, slot, &err);
    if (!P) return err;
    if (b < 0 || b > (int64_t)1 << 30) return FREEZE_EINVAL;
    if (b == 0) return FREEZE_OK;
    if (!x || !out || !workspace || (reinterpret_cast<uintptr_t>(x) % 16) != 0 ||
        (reinterpret_cast<uintptr_t>(out) % 16) != 0)
        return FREEZE_EINVAL;
    if (workspace_bytes < freeze_project_workspace_bytes(ctx, slot, b) || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return FREEZE_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const DistPlan pl = projection_plan(ctx, *P, b);
    Carver ws(workspace);
    uint16_t *x_bf = ws.take<uint16_t>((size_t)pl.b_pad * P->d_pad);
    float *tmp = ws.take<float>((size_t)b * P->n_pad);
    float *partial = pl.sk_wgs > 0 ? ws.take<float>(dist_partial_bytes(pl) / 4) : nullptr;
    if (launch_query_prep(x, nullptr, nullptr, b, pl.b_pad, pl.bm, P->d, P->d_pad, x_bf, nullptr, nullptr, nullptr, s) != hipSuccess)
        return FREEZE_EHIP;
    const bool direct = P->n == P->n_pad;   // the output rows are then exactly what the kernel writes
    DistArgs da{};
    da.q_bf = x_bf;
    da.c_bf = P->c_bf;
    da.norm = P->bias;
    da.keys = direct ? out : tmp;
    da.b = (int)b;
    da.n = (int)P->n;
    da.d_pad = (int)P->d_pad;
    da.projection = true;
    da.relu = relu != 0;
    da.partial = partial;
    if (launch_dist_topr(pl, da, s) != hipSuccess) return FREEZE_EHIP;
    if (!direct && launch_copy_rows_f32(tmp, P->n_pad, out, b, P->n, s) != hipSuccess) return FREEZE_EHIP;
    return FREEZE_OK;
}

int freeze_compact_misses(const uint8_t *hit, const int32_t *sel_in, int64_t count, int32_t *sel_out,
                          int32_t *out_count, void *stream)
{
    if (!out_count || count < 0 || count > (int64_t)1 << 30) return FREEZE_EINVAL;
    if (count > 0 && (!hit || !sel_out)) return FREEZE_EINVAL;
    if (launch_compact(hit, sel_in, nullptr, count, sel_out, out_count, nullptr, static_cast<hipStream_t>(stream)) !=
        hipSuccess)
        return FREEZE_EHIP;
    return FREEZE_OK;
}

int freeze_gather_rows(const float *x, int64_t d, const int32_t *sel, const int32_t *count, int64_t max_count,
                       float *out, void *stream)
{
    if (d < 1 || max_count < 0 || max_count > (int64_t)1 << 30) return FREEZE_EINVAL;
    if (max_count > 0 && (!x || !sel || !out)) return FREEZE_EINVAL;
    if (launch_gather_rows(x, d, sel, count, max_count, out, static_cast<hipStream_t>(stream)) != hipSuccess)
        return FREEZE_EHIP;
    return FREEZE_OK;
}

int freeze_lookup_stats_attach(freeze_ctx *ctx, void *counters)
{
    if (!ctx || (reinterpret_cast<uintptr_t>(counters) % 8) != 0) return FREEZE_EINVAL;
    ctx->stats = static_cast<unsigned long long *>(counters);
    return FREEZE_OK;
}

int freeze_profile_enable(freeze_ctx *ctx, int enable)
{
    if (!ctx) return FREEZE_EINVAL;
    if (enable < 0 || enable > 3) return FREEZE_EINVAL;
    ctx->profile = enable;
    if (enable) ctx->profile_recorded = enable == 3 ? 2 : enable;
    ctx->profiled_calls = 0;
    ctx->profile_seen = 0;
    return FREEZE_OK;
}

int freeze_profile_read(freeze_ctx *ctx, float *stage_ms, int *calls)
{
    if (!ctx || !stage_ms || !calls) return FREEZE_EINVAL;
    stage_ms[0] = stage_ms[1] = stage_ms[2] = 0.f;
    const bool light = ctx->profile_recorded == 2;   // only the distance pass was bracketed
    for (int c = 0; c < ctx->profiled_calls; ++c) {
        if (hipEventSynchronize(ctx->events[4 * c + (light ? 2 : 3)]) != hipSuccess) return FREEZE_EHIP;
        for (int i = light ? 1 : 0; i < (light ? 2 : 3); ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, ctx->events[4 * c + i], ctx->events[4 * c + i + 1]) != hipSuccess)
                return FREEZE_EHIP;
            stage_ms[i] += ms;
        }
    }
    *calls = ctx->profiled_calls;
    ctx->profiled_calls = 0;
    return FREEZE_OK;
}

int freeze_profile_read_calls(freeze_ctx *ctx, float *call_ms, int max_calls, int *calls)
{
    if (!ctx || !call_ms || !calls || max_calls < 0) return FREEZE_EINVAL;
    const int n = ctx->profiled_calls < max_calls ? ctx->profiled_calls : max_calls;
    const bool light = ctx->profile_recorded == 2;
    for (int c = 0; c < n; ++c) {
        if (hipEventSynchronize(ctx->events[4 * c + (light ? 2 : 3)]) != hipSuccess) return FREEZE_EHIP;
        for (int i = 0; i < 3; ++i) {
            call_ms[3 * c + i] = 0.f;
            if (light && i != 1) continue;
            if (hipEventElapsedTime(&call_ms[3 * c + i], ctx->events[4 * c + i], ctx->events[4 * c + i + 1]) !=
                hipSuccess)
                return FREEZE_EHIP;
        }
    }
    *calls = n;
    ctx->profiled_calls = 0;
    return FREEZE_OK;
}

const char *freeze_strerror(int code)
{
    switch (code) {
    case FREEZE_OK: return "ok";
    case FREEZE_EINVAL: return "invalid argument";
    case FREEZE_ELAYER: return "layer index out of range";
    case FREEZE_ENOTBUILT: return "layer cache not built";
    case FREEZE_EWORKSPACE: return "storage or workspace too small or misaligned";
    case FREEZE_EHIP: return "HIP runtime error";
    case FREEZE_ESCRATCH: return "look-up needs more scratch than the library's static buffer holds";
    default: return "unknown error";
    }
}

}  // extern "C"
