// Host side of the C ABI declared in include/mergecomp.h: partition policies,
// the context (segment tables, scratch, pointer-table cache), argument checks
// and the per-algorithm launch sequences.  Nothing here computes on gradient
// values; every step of the path runs in the kernels.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <limits>
#include <vector>

#include "mc_internal.h"

using namespace mc;

namespace {

constexpr uint64_t kMaxGroupElems = (1ull << 32) - (1ull << 24);
constexpr uint32_t kBarrierSpinLimit = 1u << 21;     // polls (about a microsecond each) before a block of the slow selection routes gives up waiting
constexpr int kPtrSlots = 256;           // cached device copies of per-call tensor address lists

struct Group {
    int32_t t0 = 0, t1 = 0;              // tensor range [t0, t1) of the model's list
    std::vector<int32_t> live;           // tensors of the group that hold at least one element
    uint32_t n = 0;
    uint64_t goff = 0;
    uint64_t k = 0;
    uint32_t *d_seg_off = nullptr;       // live.size() + 1 flat offsets
    uint32_t *d_chunk_seg = nullptr;     // per 1024-element chunk: tensor holding its first element
};

struct PtrSlot {
    int32_t group = -1;
    uint64_t stamp = 0;
    std::vector<uintptr_t> host;
    uintptr_t *dev = nullptr;            // tensor addresses
    uintptr_t *dev_chunk = nullptr;      // per-chunk direct addresses derived from them
};

// ---- scratch of the allocation-free entry point (mc_compress_static) ------------------------------------
// The per-tile reduction partials of the dense compressors (three arrays of one double per 4096-element tile:
// OneBit reduces two sums and a count) for groups of up to kStaticMaxElems elements, in a file-scope device
// array that every GPU the library runs on holds from the moment the code object is loaded.  The array's name
// is only a host-side handle: its device address is looked up once per device (static_scratch_for) and it is
// that pointer which the kernels receive.
constexpr uint64_t kStaticMaxElems = 1ull << 26;
constexpr size_t kStaticMaxTiles = (size_t)(kStaticMaxElems / kTile);
constexpr size_t kStaticScratchBytes = 3 * kStaticMaxTiles * sizeof(double);        // 384 KiB
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_static_mutex;
static void *g_static_ptr[kMaxDevices] = {};

// Device address of `scratch` on `device`, which must be the current device (each GPU holds its own copy of the
// array at its own address).  Looked up on the first call for a device, then served from the table.
static void *static_scratch_for(int device)
{
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[device]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        g_static_ptr[device] = ptr;
    }
    return g_static_ptr[device];
}

struct ProfEvent { int id; hipEvent_t a, b; };

struct Profiler {
    bool on = false;
    uint64_t mask = ~0ull;            // kernel slots that are timed while `on`
    std::vector<ProfEvent> pending;
    std::vector<hipEvent_t> pool;
    int64_t launches[K_COUNT] = {};
    double ms[K_COUNT] = {};
};

}  // namespace

struct mc_ctx {
    mc_config cfg{};
    int device = 0;
    std::vector<Group> groups;
    uint32_t max_tiles = 0;
    size_t max_live = 0;
    double *d_partial = nullptr;
    SparseScratch sparse{};
    uint32_t *d_hints = nullptr;        // candidate-filter hints: kHintWorkers per group (worker id modulo that)
    const uint32_t *last_hint = nullptr; // the record the most recent sparse mc_compress used (mc_select_stats)
    int *d_status = nullptr;
    void *static_scratch = nullptr;     // this device's copy of the file-scope scratch array (mc_compress_static)
    std::vector<PtrSlot> slots;
    std::vector<uintptr_t> want;        // the address list of the call in progress (reserved at creation)
    uint64_t clock = 0;
    uint32_t sync_blocks = 1;           // blocks of 1024 threads the device holds at once for sure: one per compute unit
    Profiler prof;
};

namespace mc {
static hipEvent_t prof_event(Profiler *p)
{
    hipEvent_t e = nullptr;
    if (!p->pool.empty()) { e = p->pool.back(); p->pool.pop_back(); }
    else if (hipEventCreate(&e) != hipSuccess) e = nullptr;
    return e;
}
void prof_begin(const LaunchCtx &lc, int id)
{
    Profiler *p = static_cast<Profiler *>(lc.prof);
    lc.ev_a = lc.ev_b = nullptr;
    if (!p || !p->on || !((p->mask >> id) & 1ull)) return;
    hipEvent_t a = prof_event(p), b = prof_event(p);
    if (!a || !b) {
        if (a) p->pool.push_back(a);
        if (b) p->pool.push_back(b);
        return;
    }
    lc.ev_a = a;
    lc.ev_b = b;
}
void prof_end(const LaunchCtx &lc, int id)
{
    Profiler *p = static_cast<Profiler *>(lc.prof);
    if (!p || !lc.ev_a) return;
    p->pending.push_back({id, lc.ev_a, lc.ev_b});
    lc.ev_a = lc.ev_b = nullptr;
}
}  // namespace mc

static const char *kKernelNames[K_COUNT] = {
    "upload_ptrs", "efsign_compress", "scalar_finalize", "accum_reduce", "qsgd_encode", "tern_encode",
    "fp16_compress", "dense_decompress", "sparse_accum", "sparse_seed", "cand_hist2", "cand_hist3", "cand_count",
    "cand_emit", "sparse_decompress", "state_convert", "lean_select", "lean_emit", "sparse_slow"};

static void prof_drain(Profiler &p)
{
    for (ProfEvent &e : p.pending) {
        float ms = 0.0f;
        if (hipEventSynchronize(e.b) == hipSuccess && hipEventElapsedTime(&ms, e.a, e.b) == hipSuccess) {
            p.launches[e.id] += 1;
            p.ms[e.id] += ms;
        }
        p.pool.push_back(e.a);
        p.pool.push_back(e.b);
    }
    p.pending.clear();
}

static uint64_t topk_count(uint64_t n, uint32_t ppm)
{
    if (n == 0) return 0;
    unsigned __int128 prod = (unsigned __int128)n * ppm;
    uint64_t k = (uint64_t)(prod / 1000000u);
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

// Philox-4x32-10 on the host: the sampled-threshold DGC draws where its sample starts from the word of the
// group's first element (counter = (J lo, J hi, worker, iteration), J = model-global index / 4, key = seed).
static uint32_t philox_word(uint64_t seed, uint32_t worker, uint32_t iter_lo, uint64_t global_index)
{
    const uint64_t J = global_index >> 2;
    uint32_t c[4] = {(uint32_t)J, (uint32_t)(J >> 32), worker, iter_lo};
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = 0xD2511F53ull * c[0], p1 = 0xCD9E8D57ull * c[2];
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        c[1] = (uint32_t)p1; c[3] = (uint32_t)p0; c[0] = n0; c[2] = n2;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return c[global_index & 3u];
}

// makes the context's device current for the duration of a call that synchronises or copies
struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    explicit DeviceGuard(int device)
    {
        if (hipGetDevice(&prev) == hipSuccess && prev != device) switched = hipSetDevice(device) == hipSuccess;
    }
    ~DeviceGuard() { if (switched) (void)hipSetDevice(prev); }
};

static bool is_sparse(int algo) { return algo == MC_ALGO_TOPK || algo == MC_ALGO_DGC || algo == MC_ALGO_RANDK; }
// n-element vectors of a group's state: the residual (DGC: v and u; SigNUM: the momentum; SignSGD: nothing)
static uint32_t state_vectors(int algo) { return algo == MC_ALGO_DGC ? 2u : algo == MC_ALGO_SIGNSGD ? 0u : 1u; }
static bool always_state(int algo) { return algo == MC_ALGO_DGC || algo == MC_ALGO_SIGNUM || algo == MC_ALGO_RANDK; }

extern "C" {

const char *mc_version(void) { return "mergecomp-gfx950 0.1"; }

const char *mc_strerror(int status)
{
    switch (status) {
    case MC_OK: return "ok";
    case MC_ERR_INVALID_ARG: return "invalid argument";
    case MC_ERR_RANGE: return "value out of range";
    case MC_ERR_ALLOC: return "allocation failed";
    case MC_ERR_DEVICE: return "HIP runtime error";
    case MC_ERR_PAYLOAD: return "payload header does not match the context";
    default: return "unknown status";
    }
}

int mc_partition(const int64_t *numel, int32_t n_tensors, int32_t y, int32_t policy, const int32_t *user_bounds,
                 int32_t *bounds_out)
{
    if (!numel || !bounds_out || n_tensors < 1 || y < 1) return MC_ERR_INVALID_ARG;
    for (int32_t t = 0; t < n_tensors; ++t) if (numel[t] < 0) return MC_ERR_INVALID_ARG;
    if (policy != MC_PART_EVEN_COUNT && policy != MC_PART_EVEN_ELEMS && policy != MC_PART_USER) return MC_ERR_INVALID_ARG;
    if (policy == MC_PART_USER && !user_bounds) return MC_ERR_INVALID_ARG;
    if (y > n_tensors) return MC_ERR_RANGE;
    const int32_t N = n_tensors;
    if (policy == MC_PART_EVEN_COUNT) {
        for (int32_t j = 0; j <= y; ++j) bounds_out[j] = (int32_t)(((int64_t)j * N) / y);
        return MC_OK;
    }
    if (policy == MC_PART_USER) {
        if (user_bounds[0] != 0 || user_bounds[y] != N) return MC_ERR_RANGE;
        for (int32_t j = 0; j < y; ++j) if (user_bounds[j + 1] <= user_bounds[j]) return MC_ERR_RANGE;
        std::copy(user_bounds, user_bounds + y + 1, bounds_out);
        return MC_OK;
    }
    // even by elements: one sweep over the prefix sums; boundary j is the first tensor
    // count whose prefix reaches j/y of the model, kept inside [previous + 1, N - (y - j)]
    unsigned __int128 D = 0;
    for (int32_t t = 0; t < N; ++t) D += (uint64_t)numel[t];
    bounds_out[0] = 0;
    bounds_out[y] = N;
    unsigned __int128 prefix = 0;
    int32_t t = 0;
    for (int32_t j = 1; j < y; ++j) {
        while (t < N && prefix * (unsigned)y < D * (unsigned)j) prefix += (uint64_t)numel[t++];
        int32_t b = std::min(std::max(t, bounds_out[j - 1] + 1), N - (y - j));
        bounds_out[j] = b;
    }
    return MC_OK;
}

static bool valid_model(const mc_time_model *m)
{
    return m && m->fwd_time >= 0 && m->B_h >= 0 && m->gamma_h >= 0 && m->B_g >= 0 && m->gamma_g >= 0;
}

int mc_partition_cost(const int64_t *numel, const double *bwd_time, int32_t n_tensors, const mc_time_model *model,
                      const int32_t *bounds, int32_t y, double *F_out)
{
    if (!numel || !bwd_time || !bounds || !F_out || !valid_model(model) || n_tensors < 1 || y < 1) return MC_ERR_INVALID_ARG;
    if (y > n_tensors || bounds[0] != 0 || bounds[y] != n_tensors) return MC_ERR_RANGE;
    for (int32_t j = 0; j < y; ++j) if (bounds[j + 1] <= bounds[j]) return MC_ERR_RANGE;
    double gpu = model->fwd_time, net = 0.0;
    for (int32_t j = 0; j < y; ++j) {
        double x = 0.0;
        for (int32_t t = bounds[j]; t < bounds[j + 1]; ++t) {
            if (numel[t] < 0 || bwd_time[t] < 0) return MC_ERR_INVALID_ARG;
            gpu += bwd_time[t];
            x += (double)numel[t];
        }
        gpu += model->B_h + model->gamma_h * x;
        net = std::max(gpu, net) + (model->B_g + model->gamma_g * x);
    }
    *F_out = net;
    return MC_OK;
}

int mc_partition_search(const int64_t *numel, const double *bwd_time, int32_t n_tensors, const mc_time_model *model,
                        int32_t Y, double alpha, int32_t *bounds_out, int32_t *y_out, double *F_out)
{
    if (!numel || !bwd_time || !bounds_out || !y_out || !valid_model(model) || n_tensors < 1 || Y < 1) return MC_ERR_INVALID_ARG;
    if (!(alpha >= 0.0 && alpha < 1.0)) return MC_ERR_INVALID_ARG;
    const int32_t N = n_tensors;
    if (Y > N) Y = N;
    try {
        // prefix sums over tensors: elements and back-propagation time
        std::vector<double> elems(N + 1, 0.0), bwd(N + 1, 0.0);
        for (int32_t t = 0; t < N; ++t) {
            if (numel[t] < 0 || bwd_time[t] < 0) return MC_ERR_INVALID_ARG;
            elems[t + 1] = elems[t] + (double)numel[t];
            bwd[t + 1] = bwd[t] + bwd_time[t];
        }
        // when the GPU has compressed the i-th group if that group ends before tensor e
        auto gpu_done = [&](int32_t e, int32_t i) { return model->fwd_time + bwd[e] + i * model->B_h + model->gamma_h * elems[e]; };
        auto send = [&](int32_t from, int32_t to) { return model->B_g + model->gamma_g * (elems[to] - elems[from]); };
        // net[e]: earliest time the network is free after i groups that cover tensors [0, e); from[i][e]: where the
        // last of them starts.  The time the network is free only ever delays what follows, so the earliest is best.
        const double inf = std::numeric_limits<double>::infinity();
        std::vector<double> net(N + 1, inf), next(N + 1, inf);
        std::vector<std::vector<int32_t>> from(Y + 1, std::vector<int32_t>(N + 1, 0));
        std::vector<int32_t> best_bounds, cur_bounds;
        double F_prev = 0.0;
        int32_t y_best = 1;
        for (int32_t i = 1; i <= Y; ++i) {
            std::fill(next.begin(), next.end(), inf);
            for (int32_t e = i; e <= N - 0; ++e) {
                if (i == 1) { next[e] = gpu_done(e, 1) + send(0, e); from[1][e] = 0; continue; }
                for (int32_t s0 = i - 1; s0 < e; ++s0) {
                    if (net[s0] == inf) continue;
                    const double f = std::max(gpu_done(e, i), net[s0]) + send(s0, e);
                    if (f < next[e]) { next[e] = f; from[i][e] = s0; }
                }
            }
            net.swap(next);
            const double F_now = net[N];
            cur_bounds.assign(i + 1, 0);
            cur_bounds[i] = N;
            for (int32_t j = i, e = N; j >= 1; --j) { e = from[j][e]; cur_bounds[j - 1] = e; }
            if (i == 1) { F_prev = F_now; best_bounds = cur_bounds; continue; }
            if (F_prev < F_now) break;                               // more groups made it worse: keep y - 1
            const bool stop = F_prev - F_now < alpha * F_prev;       // marginal benefit too small: keep y and stop
            F_prev = F_now; best_bounds = cur_bounds; y_best = i;
            if (stop) break;
        }
        for (int32_t j = 0; j <= y_best; ++j) bounds_out[j] = best_bounds[j];
        *y_out = y_best;
        if (F_out) *F_out = F_prev;
    } catch (const std::bad_alloc &) {
        return MC_ERR_ALLOC;
    }
    return MC_OK;
}

int mc_ctx_destroy(mc_ctx *ctx)
{
    if (!ctx) return MC_ERR_INVALID_ARG;
    int prev = 0;
    bool switched = hipGetDevice(&prev) == hipSuccess && prev != ctx->device && hipSetDevice(ctx->device) == hipSuccess;
    (void)hipDeviceSynchronize();
    prof_drain(ctx->prof);
    for (hipEvent_t e : ctx->prof.pool) (void)hipEventDestroy(e);
    for (Group &g : ctx->groups) {
        if (g.d_seg_off) (void)hipFree(g.d_seg_off);
        if (g.d_chunk_seg) (void)hipFree(g.d_chunk_seg);
    }
    for (PtrSlot &s : ctx->slots) {
        if (s.dev) (void)hipFree(s.dev);
        if (s.dev_chunk) (void)hipFree(s.dev_chunk);
    }
    if (ctx->d_partial) (void)hipFree(ctx->d_partial);
    void *sparse_bufs[] = {ctx->sparse.hist, ctx->sparse.sel, ctx->d_hints, ctx->sparse.cand_bits, ctx->sparse.cand_loc,
                           ctx->sparse.tile_runs, ctx->sparse.tile_cnt, ctx->sparse.blk_cnt, ctx->sparse.ulist, ctx->sparse.ucount,
                           ctx->sparse.sync};
    for (void *b : sparse_bufs) if (b) (void)hipFree(b);
    if (ctx->d_status) (void)hipFree(ctx->d_status);
    if (switched) (void)hipSetDevice(prev);
    delete ctx;
    return MC_OK;
}

int mc_ctx_create(mc_ctx **out, const mc_config *cfg, const int64_t *numel, int32_t n_tensors, const int32_t *bounds,
                  int32_t y)
{
    if (!out) return MC_ERR_INVALID_ARG;
    *out = nullptr;
    if (!cfg || !numel || !bounds || n_tensors < 1 || y < 1) return MC_ERR_INVALID_ARG;
    if (cfg->algo < MC_ALGO_EFSIGN || cfg->algo > MC_ALGO_RANDK) return MC_ERR_INVALID_ARG;
    if (cfg->dgc_sample_ppm > 1000000u || (cfg->dgc_sample_ppm != 0 && cfg->algo != MC_ALGO_DGC)) return MC_ERR_INVALID_ARG;
    if (cfg->use_ef != 0 && cfg->use_ef != 1) return MC_ERR_INVALID_ARG;
    if (always_state(cfg->algo) && cfg->use_ef != 1) return MC_ERR_INVALID_ARG;
    if (cfg->algo == MC_ALGO_SIGNSGD && cfg->use_ef != 0) return MC_ERR_INVALID_ARG;
    if (cfg->algo == MC_ALGO_QSGD && (cfg->qsgd_bits < 2 || cfg->qsgd_bits > 8)) return MC_ERR_INVALID_ARG;
    if (is_sparse(cfg->algo) && (cfg->ratio_ppm < 1 || cfg->ratio_ppm > 1000000u)) return MC_ERR_INVALID_ARG;
    if (y > n_tensors) return MC_ERR_RANGE;
    if (bounds[0] != 0 || bounds[y] != n_tensors) return MC_ERR_RANGE;
    for (int32_t j = 0; j < y; ++j) if (bounds[j + 1] <= bounds[j]) return MC_ERR_RANGE;
    for (int32_t t = 0; t < n_tensors; ++t) if (numel[t] < 0) return MC_ERR_INVALID_ARG;
    for (int32_t j = 0; j < y; ++j) {      // flat indices of a group are 32-bit
        uint64_t n = 0;
        for (int32_t t = bounds[j]; t < bounds[j + 1]; ++t) {
            if ((uint64_t)numel[t] >= kMaxGroupElems) return MC_ERR_RANGE;
            n += (uint64_t)numel[t];
            if (n >= kMaxGroupElems) return MC_ERR_RANGE;
        }
    }

    mc_ctx *ctx = new (std::nothrow) mc_ctx();
    if (!ctx) return MC_ERR_ALLOC;
    ctx->cfg = *cfg;
    if (hipGetDevice(&ctx->device) != hipSuccess) { delete ctx; return MC_ERR_DEVICE; }
    int rc = MC_OK;
    try {
        ctx->groups.resize(y);
        uint64_t goff = 0;
        for (int32_t j = 0; j < y && rc == MC_OK; ++j) {
            Group &g = ctx->groups[j];
            g.t0 = bounds[j]; g.t1 = bounds[j + 1]; g.goff = goff;
            std::vector<uint32_t> off;
            uint64_t n = 0;
            for (int32_t t = g.t0; t < g.t1; ++t) {
                if (numel[t] == 0) continue;
                g.live.push_back(t - g.t0);
                off.push_back((uint32_t)n);
                n += (uint64_t)numel[t];
            }
            off.push_back((uint32_t)n);
            g.n = (uint32_t)n;
            g.k = is_sparse(cfg->algo) ? topk_count(n, cfg->ratio_ppm) : 0;
            if (cfg->dgc_sample_ppm) g.k = std::min<uint64_t>(2 * g.k, n);     // sampled threshold: the payload's capacity
            goff += n;
            if (hipMalloc(&g.d_seg_off, off.size() * sizeof(uint32_t)) != hipSuccess) { rc = MC_ERR_ALLOC; break; }
            if (hipMemcpy(g.d_seg_off, off.data(), off.size() * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess) { rc = MC_ERR_DEVICE; break; }
            std::vector<uint32_t> cseg((size_t)((n + kChunk - 1) / kChunk) + 1, 0u);
            for (size_t c = 0, sidx = 0; c * kChunk < n; ++c) {
                while (off[sidx + 1] <= c * kChunk) ++sidx;
                cseg[c] = (uint32_t)sidx;
            }
            if (hipMalloc(&g.d_chunk_seg, cseg.size() * sizeof(uint32_t)) != hipSuccess) { rc = MC_ERR_ALLOC; break; }
            if (hipMemcpy(g.d_chunk_seg, cseg.data(), cseg.size() * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess) { rc = MC_ERR_DEVICE; break; }
            ctx->max_tiles = std::max<uint32_t>(ctx->max_tiles, (uint32_t)((n + kTile - 1) / kTile));
            ctx->max_live = std::max(ctx->max_live, g.live.size());
        }
        const size_t tiles = std::max<size_t>(ctx->max_tiles, 1);
        if (rc == MC_OK && hipMalloc(&ctx->d_partial, 3 * tiles * sizeof(double)) != hipSuccess) rc = MC_ERR_ALLOC;
        if (rc == MC_OK && hipMalloc(&ctx->d_status, sizeof(int)) != hipSuccess) rc = MC_ERR_ALLOC;
        if (rc == MC_OK && hipMemset(ctx->d_status, 0, sizeof(int)) != hipSuccess) rc = MC_ERR_DEVICE;
        if (rc == MC_OK && is_sparse(cfg->algo)) {
            SparseScratch &sp = ctx->sparse;
            const size_t hist_bytes = kHistWords * sizeof(uint32_t);
            const size_t chunks = tiles * kWavesPerBlock, slots = chunks * kChunk;
            if (hipMalloc(&sp.hist, hist_bytes) != hipSuccess || hipMalloc(&sp.sel, 4 * sizeof(SelectState)) != hipSuccess ||
                hipMalloc(&ctx->d_hints, (size_t)y * kHintWorkers * kHintWords * sizeof(uint32_t)) != hipSuccess ||
                hipMalloc(&sp.cand_bits, slots * sizeof(uint32_t)) != hipSuccess ||
                hipMalloc(&sp.cand_loc, slots * sizeof(uint16_t)) != hipSuccess ||
                hipMalloc(&sp.tile_runs, tiles * sizeof(uint64_t)) != hipSuccess ||
                hipMalloc(&sp.tile_cnt, tiles * sizeof(uint32_t)) != hipSuccess ||
                hipMalloc(&sp.blk_cnt, (tiles + kWavesPerBlock - 1) / kWavesPerBlock * sizeof(uint32_t)) != hipSuccess ||
                hipMalloc(&sp.ulist, (size_t)kUSub * kUCap * sizeof(UEntry)) != hipSuccess ||
                hipMalloc(&sp.ucount, (size_t)kUSub * kUCountStride * sizeof(uint32_t)) != hipSuccess ||
                hipMalloc(&sp.sync, 64 * sizeof(uint32_t)) != hipSuccess) rc = MC_ERR_ALLOC;
            else if (hipMemset(sp.hist, 0, hist_bytes) != hipSuccess || hipMemset(sp.sel, 0, 4 * sizeof(SelectState)) != hipSuccess ||
                     hipMemset(ctx->d_hints, 0, (size_t)y * kHintWorkers * kHintWords * sizeof(uint32_t)) != hipSuccess ||
                     hipMemset(sp.tile_runs, 0, tiles * sizeof(uint64_t)) != hipSuccess ||
                     hipMemset(sp.ucount, 0, (size_t)kUSub * kUCountStride * sizeof(uint32_t)) != hipSuccess ||
                     hipMemset(sp.sync, 0, 64 * sizeof(uint32_t)) != hipSuccess) rc = MC_ERR_DEVICE;
            int cus = 0;
            if (rc == MC_OK && (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device) != hipSuccess || cus < 1)) rc = MC_ERR_DEVICE;
            ctx->sync_blocks = (uint32_t)std::max(cus, 1);
            sp.spin_limit = kBarrierSpinLimit;
        }
        if (rc == MC_OK) {
            // the per-chunk address tables of all slots together stay below 256 MiB
            const size_t per_slot = tiles * kWavesPerBlock * sizeof(uintptr_t);
            ctx->slots.resize(std::min<size_t>(kPtrSlots, std::max<size_t>(4, (size_t(256) << 20) / per_slot)));
            for (PtrSlot &s : ctx->slots) {
                if (hipMalloc(&s.dev, std::max<size_t>(ctx->max_live, 1) * sizeof(uintptr_t)) != hipSuccess ||
                    hipMalloc(&s.dev_chunk, tiles * kWavesPerBlock * sizeof(uintptr_t)) != hipSuccess) { rc = MC_ERR_ALLOC; break; }
                s.host.reserve(ctx->max_live);
            }
            ctx->want.reserve(ctx->max_live);
            ctx->prof.pending.reserve(1024);
            ctx->prof.pool.reserve(2048);
        }
        // the device address of the static scratch array, looked up here with the context's device current
        if (rc == MC_OK && !(ctx->static_scratch = static_scratch_for(ctx->device))) rc = MC_ERR_DEVICE;
        if (rc == MC_OK && hipDeviceSynchronize() != hipSuccess) rc = MC_ERR_DEVICE;
    } catch (const std::bad_alloc &) {
        rc = MC_ERR_ALLOC;
    }
    if (rc != MC_OK) { mc_ctx_destroy(ctx); return rc; }
    *out = ctx;
    return MC_OK;
}

static const Group *group_of(const mc_ctx *ctx, int32_t group)
{
    if (!ctx || group < 0 || (size_t)group >= ctx->groups.size()) return nullptr;
    return &ctx->groups[group];
}

int64_t mc_group_numel(const mc_ctx *ctx, int32_t group) { const Group *g = group_of(ctx, group); return g ? (int64_t)g->n : -1; }
int64_t mc_group_k(const mc_ctx *ctx, int32_t group) { const Group *g = group_of(ctx, group); return g ? (int64_t)g->k : -1; }
int32_t mc_group_tensors(const mc_ctx *ctx, int32_t group) { const Group *g = group_of(ctx, group); return g ? g->t1 - g->t0 : -1; }

size_t mc_payload_bytes(const mc_ctx *ctx, int32_t group)
{
    const Group *g = group_of(ctx, group);
    if (!g) return 0;
    const uint64_t n = g->n, words = (n + 31) / 32;
    switch (ctx->cfg.algo) {
    case MC_ALGO_EFSIGN:
    case MC_ALGO_ONEBIT:
    case MC_ALGO_SIGNSGD:
    case MC_ALGO_SIGNUM: return kHeaderBytes + 4 * words;
    case MC_ALGO_TERNGRAD: return kHeaderBytes + 8 * words;
    case MC_ALGO_QSGD: return kHeaderBytes + (n + 3) / 4 * 4;
    case MC_ALGO_FP16: return kHeaderBytes + (2 * n + 3) / 4 * 4;
    default: return kHeaderBytes + 8 * g->k + (n ? 4 * ((n + kTile - 1) / kTile + 1) : 0);      // index and value lists, directory
    }
}

size_t mc_state_bytes(const mc_ctx *ctx, int32_t group)
{
    const Group *g = group_of(ctx, group);
    if (!g) return 0;
    if (ctx->cfg.algo == MC_ALGO_DGC) return kHeaderBytes + sizeof(float) * (dgc_u_offset(g->n) + (size_t)g->n);
    return kHeaderBytes + sizeof(float) * (size_t)g->n * state_vectors(ctx->cfg.algo);
}

// Device view of a group over a per-call tensor address list (only tensors that hold
// elements).  Lists seen before are served from the cache; a new list replaces the
// least recently used slot: it is uploaded through a kernel's argument buffer and
// expanded into the per-chunk address table, in stream order with the kernels that
// will read it.
static GroupView group_view(mc_ctx *ctx, const LaunchCtx &lc, int32_t group, const Group &g, const void *const *ptrs)
{
    std::vector<uintptr_t> &want = ctx->want;     // capacity max_live: no allocation here
    want.clear();
    for (int32_t rel : g.live) want.push_back(reinterpret_cast<uintptr_t>(ptrs[rel]));
    GroupView gv{g.d_seg_off, g.d_chunk_seg, nullptr, nullptr, (uint32_t)g.live.size(), g.n, g.goff};
    PtrSlot *victim = &ctx->slots[0];
    for (PtrSlot &s : ctx->slots) {
        if (s.group == group && s.host.size() == want.size() &&
            std::memcmp(s.host.data(), want.data(), want.size() * sizeof(uintptr_t)) == 0) {
            s.stamp = ++ctx->clock;
            gv.ptrs = s.dev;
            gv.chunk_addr = s.dev_chunk;
            return gv;
        }
        if (s.stamp < victim->stamp) victim = &s;
    }
    victim->group = group;
    victim->stamp = ++ctx->clock;
    victim->host = want;
    gv.ptrs = victim->dev;
    gv.chunk_addr = victim->dev_chunk;
    if (!want.empty()) {
        launch_upload_ptrs(lc, want.data(), victim->dev, (uint32_t)want.size());
        launch_expand_ptrs(lc, gv, victim->dev_chunk);
    }
    return gv;
}

static int check_launch() { return hipGetLastError() == hipSuccess ? MC_OK : MC_ERR_DEVICE; }

// partial: the per-tile reduction partials (three arrays of one double per tile of the group); prof: the context's
// profiler, or null for a call that must not create events
static int compress_impl(mc_ctx *ctx, int32_t group, uint32_t worker, uint64_t iter, const float *const *grad_ptrs, void *state,
                         void *payload_out, void *stream, double *partial, Profiler *prof)
{
    const Group *gp = group_of(ctx, group);
    if (!gp || !payload_out) return MC_ERR_INVALID_ARG;
    const Group &G = *gp;
    const mc_config &cfg = ctx->cfg;
    const bool ef = cfg.use_ef != 0;
    if (ef && !state) return MC_ERR_INVALID_ARG;
    if (G.t1 > G.t0 && !grad_ptrs) return MC_ERR_INVALID_ARG;
    for (int32_t rel : G.live) if (!grad_ptrs[rel] || (reinterpret_cast<uintptr_t>(grad_ptrs[rel]) & 3u)) return MC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(payload_out) & 15u) || (reinterpret_cast<uintptr_t>(state) & 15u)) return MC_ERR_INVALID_ARG;

    LaunchCtx lc{static_cast<hipStream_t>(stream), prof, nullptr, nullptr};
    (void)hipGetLastError();
    PayloadHeader *hdr = static_cast<PayloadHeader *>(payload_out);
    uint8_t *body = static_cast<uint8_t *>(payload_out) + kHeaderBytes;
    StateHeader *sh = static_cast<StateHeader *>(state);
    float *sf = state ? reinterpret_cast<float *>(static_cast<uint8_t *>(state) + kHeaderBytes) : nullptr;
    const uint32_t n = G.n, nwords = (uint32_t)(((uint64_t)n + 31) / 32);
    const uint32_t tiles = (uint32_t)(((uint64_t)n + kTile - 1) / kTile);
    const uint32_t levels = cfg.algo == MC_ALGO_QSGD ? (1u << (cfg.qsgd_bits - 1)) - 1u : 0u;

    if (n == 0) {   // nothing to encode: the payload is its header
        const bool votes = cfg.algo == MC_ALGO_SIGNSGD || cfg.algo == MC_ALGO_SIGNUM;
        launch_scalar_finalize(lc, partial, 0, votes ? RED_ONE : -1, 0, hdr, (uint32_t)cfg.algo, 0, levels, nullptr);
        return check_launch();
    }
    GroupView gv = group_view(ctx, lc, group, G, reinterpret_cast<const void *const *>(grad_ptrs));
    switch (cfg.algo) {
    case MC_ALGO_EFSIGN:
        launch_sign_compress(lc, SIGN_EF, gv, ef, sf, sh, 0.0f, reinterpret_cast<uint32_t *>(body), nwords, partial, hdr, MC_ALGO_EFSIGN);
        launch_scalar_finalize(lc, partial, tiles, RED_MEAN_ABS, n, hdr, MC_ALGO_EFSIGN, 0, 0, ef ? &sh->scale : nullptr);
        break;
    case MC_ALGO_ONEBIT:
        launch_sign_compress(lc, SIGN_MEANS, gv, ef, sf, sh, 0.0f, reinterpret_cast<uint32_t *>(body), nwords, partial, hdr, MC_ALGO_ONEBIT);
        launch_scalar_finalize(lc, partial, tiles, RED_MEANS, n, hdr, MC_ALGO_ONEBIT, 0, 0, ef ? &sh->scale : nullptr);
        break;
    case MC_ALGO_SIGNSGD:
    case MC_ALGO_SIGNUM:
        launch_sign_compress(lc, cfg.algo == MC_ALGO_SIGNSGD ? SIGN_PLAIN : SIGN_MOMENTUM, gv, ef, sf, sh, cfg.dgc_momentum,
                             reinterpret_cast<uint32_t *>(body), nwords, partial, hdr, (uint32_t)cfg.algo);
        break;
    case MC_ALGO_QSGD:
        launch_accum_reduce(lc, gv, ef, sf, sh, RED_L2, levels, cfg.seed, partial);
        launch_scalar_finalize(lc, partial, tiles, RED_L2, n, hdr, MC_ALGO_QSGD, 0, levels, nullptr);
        launch_qsgd_encode(lc, gv, ef, sf, sh, hdr, reinterpret_cast<int8_t *>(body), levels, cfg.seed, worker, (uint32_t)iter);
        break;
    case MC_ALGO_TERNGRAD:
        launch_accum_reduce(lc, gv, ef, sf, sh, RED_MAX_ABS, 0, cfg.seed, partial);
        launch_scalar_finalize(lc, partial, tiles, RED_MAX_ABS, n, hdr, MC_ALGO_TERNGRAD, 0, 0, nullptr);
        launch_tern_encode(lc, gv, ef, sf, sh, hdr, reinterpret_cast<uint32_t *>(body), nwords, cfg.seed, worker, (uint32_t)iter);
        break;
    case MC_ALGO_FP16:
        launch_fp16_compress(lc, gv, ef, sf, hdr, reinterpret_cast<uint16_t *>(body));
        break;
    case MC_ALGO_TOPK:
    case MC_ALGO_DGC:
    case MC_ALGO_RANDK:
    {
        SparseScratch sp = ctx->sparse;
        // a context may compress for several simulated workers whose thresholds differ: each keeps its own hint
        sp.hint = ctx->d_hints + ((size_t)group * kHintWorkers + worker % kHintWorkers) * kHintWords;
        ctx->last_hint = sp.hint;
        uint32_t stride = 0, first = 0;
        uint64_t need = 0;
        if (cfg.dgc_sample_ppm) {       // sample: every stride-th element from `first`; threshold = its need-th largest key
            stride = std::max<uint32_t>(1u, 1000000u / cfg.dgc_sample_ppm);
            first = philox_word(cfg.seed, worker, (uint32_t)iter, G.goff) % stride;
            const uint64_t m = n > first ? ((uint64_t)n - first + stride - 1) / stride : 0;
            need = m ? std::max<uint64_t>(1, (uint64_t)(((unsigned __int128)m * cfg.ratio_ppm) / 1000000u)) : 0;
        }
        launch_sparse_compress(lc, cfg.algo, gv, ef, sf, cfg.dgc_momentum, G.k, hdr, sp, cfg.seed, worker, (uint32_t)iter,
                               stride, first, need, ctx->sync_blocks, ctx->d_status);
    }
        break;
    default: return MC_ERR_INVALID_ARG;
    }
    return check_launch();
}

int mc_compress(mc_ctx *ctx, int32_t group, uint32_t worker, uint64_t iter, const float *const *grad_ptrs, void *state,
                void *payload_out, void *stream)
{
    if (!ctx) return MC_ERR_INVALID_ARG;
    return compress_impl(ctx, group, worker, iter, grad_ptrs, state, payload_out, stream, ctx->d_partial, &ctx->prof);
}

int mc_compress_static(mc_ctx *ctx, int32_t group, uint32_t worker, uint64_t iter, const float *const *grad_ptrs, void *state,
                       void *payload_out, void *stream)
{
    const Group *gp = group_of(ctx, group);
    if (!gp) return MC_ERR_INVALID_ARG;
    // the sparsifiers' scratch (candidate slots, 6 bytes per element) is not what the static array holds
    if (is_sparse(ctx->cfg.algo)) return MC_ERR_INVALID_ARG;
    if ((uint64_t)gp->n > kStaticMaxElems) return MC_ERR_RANGE;
    if (!ctx->static_scratch) return MC_ERR_DEVICE;
    // every tile's partial is written by the compress kernel before the one-block combine reads it: nothing in the
    // array has to start at zero, whatever an earlier call left there
    return compress_impl(ctx, group, worker, iter, grad_ptrs, state, payload_out, stream,
                         static_cast<double *>(ctx->static_scratch), nullptr);
}

size_t mc_static_scratch_bytes(void) { return kStaticScratchBytes; }
int64_t mc_static_max_elems(void) { return (int64_t)kStaticMaxElems; }

int mc_decompress_sum(mc_ctx *ctx, int32_t group, const void *const *payloads, int32_t W, float alpha,
                      float *const *out_ptrs, void *stream)
{
    const Group *gp = group_of(ctx, group);
    if (!gp || !payloads || W < 1) return MC_ERR_INVALID_ARG;
    if (W > kMaxWorkers) return MC_ERR_RANGE;
    const Group &G = *gp;
    if (G.t1 > G.t0 && !out_ptrs) return MC_ERR_INVALID_ARG;
    for (int32_t rel : G.live) if (!out_ptrs[rel] || (reinterpret_cast<uintptr_t>(out_ptrs[rel]) & 3u)) return MC_ERR_INVALID_ARG;
    PayloadPtrs pl{};
    for (int32_t w = 0; w < W; ++w) {
        if (!payloads[w] || (reinterpret_cast<uintptr_t>(payloads[w]) & 15u)) return MC_ERR_INVALID_ARG;
        pl.p[w] = static_cast<const uint8_t *>(payloads[w]);
    }
    if (G.n == 0) return MC_OK;
    LaunchCtx lc{static_cast<hipStream_t>(stream), &ctx->prof, nullptr, nullptr};
    (void)hipGetLastError();
    GroupView gv = group_view(ctx, lc, group, G, reinterpret_cast<const void *const *>(out_ptrs));
    const mc_config &cfg = ctx->cfg;
    if (is_sparse(cfg.algo)) launch_sparse_decompress(lc, cfg.algo, gv, pl, W, alpha, G.k, ctx->d_status, cfg.dgc_sample_ppm != 0);
    else {
        const uint32_t levels = cfg.algo == MC_ALGO_QSGD ? (1u << (cfg.qsgd_bits - 1)) - 1u : 0u;
        launch_dense_decompress(lc, cfg.algo, gv, pl, W, alpha, levels, ctx->d_status);
    }
    return check_launch();
}

int mc_compress_groups(mc_ctx *ctx, uint32_t worker, uint64_t iter, const float *const *grad_ptrs_all, void *const *states,
                       void *const *payloads_out, void *stream)
{
    if (!ctx || !payloads_out || (ctx->cfg.use_ef && !states)) return MC_ERR_INVALID_ARG;
    for (size_t j = 0; j < ctx->groups.size(); ++j) {
        const Group &G = ctx->groups[j];
        const int rc = compress_impl(ctx, (int32_t)j, worker, iter, grad_ptrs_all ? grad_ptrs_all + G.t0 : nullptr, states ? states[j] : nullptr,
                                     payloads_out[j], stream, ctx->d_partial, &ctx->prof);
        if (rc != MC_OK) return rc;
    }
    return MC_OK;
}

int mc_decompress_sum_groups(mc_ctx *ctx, const void *const *payloads, int32_t W, float alpha, float *const *out_ptrs_all, void *stream)
{
    if (!ctx || !payloads || W < 1) return MC_ERR_INVALID_ARG;
    if (W > kMaxWorkers) return MC_ERR_RANGE;
    const size_t y = ctx->groups.size();
    const void *one[kMaxWorkers];
    for (size_t j = 0; j < y; ++j) {
        for (int32_t w = 0; w < W; ++w) one[w] = payloads[(size_t)w * y + j];
        const int rc = mc_decompress_sum(ctx, (int32_t)j, one, W, alpha, out_ptrs_all ? out_ptrs_all + ctx->groups[j].t0 : nullptr, stream);
        if (rc != MC_OK) return rc;
    }
    return MC_OK;
}

static int state_convert(mc_ctx *ctx, int32_t group, const void *src, void *dst, bool to_residual, void *stream)
{
    const Group *g = group_of(ctx, group);
    if (!g) return MC_ERR_INVALID_ARG;
    const size_t nf = (size_t)g->n * state_vectors(ctx->cfg.algo);
    // an empty group has no residual: the plain side may be null, the opaque side never
    if (!(to_residual ? src : dst) || (nf > 0 && !(to_residual ? dst : src))) return MC_ERR_INVALID_ARG;
    // Nothing to convert (an empty group, or SignSGD, which keeps no state vector): neither side is touched.  The
    // kernel below indexes by the group's n, so it must never run for an algorithm without state vectors.
    if (nf == 0) return MC_OK;
    LaunchCtx lc{static_cast<hipStream_t>(stream), &ctx->prof, nullptr, nullptr};
    (void)hipGetLastError();
    const uint32_t levels = ctx->cfg.algo == MC_ALGO_QSGD ? (1u << (ctx->cfg.qsgd_bits - 1)) - 1u : 0u;
    launch_state_convert(lc, ctx->cfg.algo, to_residual, g->n, src, dst, levels, ctx->cfg.seed, g->goff);
    return check_launch();
}

int mc_state_export_residual(mc_ctx *ctx, int32_t group, const void *state, float *e_out, void *stream)
{
    return state_convert(ctx, group, state, e_out, true, stream);
}

int mc_state_import_residual(mc_ctx *ctx, int32_t group, const float *e_in, void *state, void *stream)
{
    return state_convert(ctx, group, e_in, state, false, stream);
}

int mc_last_device_status(mc_ctx *ctx)
{
    if (!ctx) return MC_ERR_INVALID_ARG;
    int flag = 0;
    DeviceGuard on(ctx->device);
    if (hipDeviceSynchronize() != hipSuccess) return MC_ERR_DEVICE;
    if (hipMemcpy(&flag, ctx->d_status, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return MC_ERR_DEVICE;
    if (flag && hipMemset(ctx->d_status, 0, sizeof(int)) != hipSuccess) return MC_ERR_DEVICE;
    return flag == 2 ? MC_ERR_DEVICE : flag ? MC_ERR_PAYLOAD : MC_OK;
}

int mc_last_select_route(mc_ctx *ctx)
{
    if (!ctx || !is_sparse(ctx->cfg.algo) || !ctx->sparse.sel) return MC_ERR_INVALID_ARG;
    SelectState s;
    DeviceGuard on(ctx->device);
    if (hipDeviceSynchronize() != hipSuccess) return MC_ERR_DEVICE;
    if (hipMemcpy(&s, ctx->sparse.sel, sizeof(s), hipMemcpyDeviceToHost) != hipSuccess) return MC_ERR_DEVICE;
    return (s.mode & 8u) ? MC_SELECT_DENSE : (s.mode & 1u) ? MC_SELECT_FAST : (s.mode & 2u) ? MC_SELECT_REFILL : MC_SELECT_ABOVE;
}

int mc_select_stats(mc_ctx *ctx, mc_select_counts *out, int32_t reset)
{
    if (!ctx || !out || !is_sparse(ctx->cfg.algo) || !ctx->sparse.sync) return MC_ERR_INVALID_ARG;
    uint32_t w[16] = {};
    DeviceGuard on(ctx->device);
    if (hipDeviceSynchronize() != hipSuccess) return MC_ERR_DEVICE;
    if (hipMemcpy(w, ctx->sparse.sync + 32, sizeof(w), hipMemcpyDeviceToHost) != hipSuccess) return MC_ERR_DEVICE;
    for (int r = 0; r < 4; ++r) out->calls[r] = w[r];
    out->last_bin_keys = w[8];
    out->last_candidates = w[9];
    out->margin_halvings = out->margin_cap = -1;
    if (ctx->last_hint) {
        uint32_t h[kHintWords] = {};
        if (hipMemcpy(h, ctx->last_hint, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return MC_ERR_DEVICE;
        out->margin_halvings = h[1];
        out->margin_cap = 4 - (int64_t)std::min<uint32_t>(h[3] & 0xFFu, 4u);
    }
    if (reset && hipMemset(ctx->sparse.sync + 32, 0, 4 * sizeof(uint32_t)) != hipSuccess) return MC_ERR_DEVICE;
    return MC_OK;
}

int mc_set_barrier_spin_limit(mc_ctx *ctx, uint32_t polls)
{
    if (!ctx || !is_sparse(ctx->cfg.algo)) return MC_ERR_INVALID_ARG;
    ctx->sparse.spin_limit = polls ? polls - 1u : kBarrierSpinLimit;       // polls = 1: give up after the first look
    return MC_OK;
}

int mc_profile_enable(mc_ctx *ctx, int32_t on)
{
    if (!ctx) return MC_ERR_INVALID_ARG;
    ctx->prof.on = on != 0;
    return MC_OK;
}

int mc_profile_select(mc_ctx *ctx, uint64_t kernel_mask)
{
    if (!ctx) return MC_ERR_INVALID_ARG;
    ctx->prof.mask = kernel_mask;
    return MC_OK;
}

int mc_profile_reset(mc_ctx *ctx)
{
    if (!ctx) return MC_ERR_INVALID_ARG;
    prof_drain(ctx->prof);
    for (int i = 0; i < K_COUNT; ++i) { ctx->prof.launches[i] = 0; ctx->prof.ms[i] = 0.0; }
    return MC_OK;
}

int32_t mc_profile_kernels(void) { return K_COUNT; }

int mc_profile_read(mc_ctx *ctx, int32_t id, const char **name, int64_t *launches, double *total_ms)
{
    if (!ctx || id < 0 || id >= K_COUNT) return MC_ERR_INVALID_ARG;
    prof_drain(ctx->prof);
    if (name) *name = kKernelNames[id];
    if (launches) *launches = ctx->prof.launches[id];
    if (total_ms) *total_ms = ctx->prof.ms[id];
    return MC_OK;
}

}  // extern "C"
