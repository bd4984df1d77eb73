// Sparsifiers (Top-k, DGC) for gfx950: exact top-k of |p| over a whole merged
// group by radix select on the fp32 bit pattern, ties at the threshold taken in
// index order (lower index wins), payload written in ascending index order, and
// the sparse decompress-and-sum.
//
// The paper singles out the top-k() operation as the cost that merging alone
// does not remove (Section 5.1).  Here it is a three-level histogram
// (11 + 10 + 10 bits of the 31-bit magnitude key) followed by an ordered
// compaction, all on the merged group, so the selection is one operation per
// group however many tensors the group has.
//
// Kernels of one compress call (all on the caller's stream, no host sync):
//   accumulate   p = g + e (DGC: u = m u + g, v = v + u), kept in the state; level-1 histogram
//   select_bin   one block: locate the bin that holds the k-th largest key, narrow `need`
//   hist         level-2 / level-3 histograms of the keys that match the prefix so far
//   count        per tile: keys above / equal to the threshold
//   scan         one block: exclusive prefix of the per-tile counts
//   emit         ordered compaction into (idx, val); selected entries leave the residual
#include "mc_internal.h"

namespace mc {

static inline uint32_t tiles_of(uint32_t n) { return (uint32_t)(((uint64_t)n + kTile - 1) / kTile); }

constexpr int kBins1 = 2048, kBins2 = 1024, kBins3 = 1024;

__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// ---------------------------------------------------------------------------
// accumulate + level-1 histogram
// ---------------------------------------------------------------------------
template <int ALGO, bool EF>
__global__ __launch_bounds__(kBlock) void sparse_accum_k(GroupView g, float *st, float momentum, uint32_t *ghist)
{
    __shared__ uint32_t hist[kBins1];
    for (int b = threadIdx.x; b < kBins1; b += kBlock) hist[b] = 0u;
    __syncthreads();
    const Chunk c = my_chunk(g.n);
    if (c.base < g.n) {
        float p[kSteps];
        load_seg(g, c, p);
        if (ALGO == MC_ALGO_DGC) {
            // momentum correction: u = m u + g ; v = v + u ; the vector compressed is v
            float *vbuf = st, *ubuf = st + g.n;
            float u[kSteps], v[kSteps];
            load_flat(ubuf, c, g.n, u, 0.0f);
            load_flat(vbuf, c, g.n, v, 0.0f);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                float mu = momentum * u[j];
                u[j] = mu + p[j];
                v[j] = v[j] + u[j];
                p[j] = v[j];
            }
            store_flat(ubuf, c, g.n, u);
            store_flat(vbuf, c, g.n, v);
        } else if (EF) {
            float e[kSteps];
            load_flat(st, c, g.n, e, 0.0f);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) p[j] = p[j] + e[j];
            store_flat(st, c, g.n, p);
        }
#pragma unroll
        for (int j = 0; j < kSteps; ++j)
            if (c.full || c.base + 64 * j + c.lane < g.n) atomicAdd(&hist[key_of(p[j]) >> 20], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins1; b += kBlock) {
        uint32_t h = hist[b];
        if (h) atomicAdd(&ghist[b], h);
    }
}

// the vector the later passes select from: v / p kept in the state, or the gradient itself
template <bool FROM_STATE>
__device__ __forceinline__ void load_sel(const GroupView &g, const float *st, const Chunk &c, float (&p)[kSteps])
{
    if (FROM_STATE) load_flat(st, c, g.n, p, 0.0f);
    else load_seg(g, c, p);
}

// ---------------------------------------------------------------------------
// one block: find the bin b with  count(bins > b) < need <= count(bins >= b),
// append it to the prefix, reduce need by count(bins > b), clear the histogram
// ---------------------------------------------------------------------------
template <int BINS>
__global__ __launch_bounds__(kBlock) void select_bin_k(uint32_t *hist, SelectState *sel, int first, uint64_t k, int shift)
{
    constexpr int kPer = BINS / kBlock;
    __shared__ uint64_t above[kBlock];
    const int t = threadIdx.x;
    uint32_t h[kPer];
    uint64_t own = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) { h[i] = hist[t * kPer + i]; own += h[i]; hist[t * kPer + i] = 0u; }
    // inclusive suffix sum over threads (thread 255 owns the highest bins)
    above[t] = own;
    __syncthreads();
    for (int d = 1; d < kBlock; d <<= 1) {
        uint64_t add = t + d < kBlock ? above[t + d] : 0;
        __syncthreads();
        above[t] += add;
        __syncthreads();
    }
    const uint64_t need = first ? k : sel->need;
    const uint32_t prefix = first ? 0u : sel->prefix;
    __syncthreads();
    uint64_t run = above[t] - own;                 // keys in bins owned by higher threads
    if (run < need && need <= run + own) {
#pragma unroll
        for (int i = kPer - 1; i >= 0; --i) {
            if (run < need && need <= run + h[i]) {
                sel->prefix = prefix | ((uint32_t)(t * kPer + i) << shift);
                sel->need = need - run;
            }
            run += h[i];
        }
    }
}

// ---------------------------------------------------------------------------
// level-2 / level-3 histogram of the keys whose upper bits equal the prefix
// ---------------------------------------------------------------------------
template <bool FROM_STATE, int LEVEL>
__global__ __launch_bounds__(kBlock) void sparse_hist_k(GroupView g, const float *st, const SelectState *sel, uint32_t *ghist)
{
    __shared__ uint32_t hist[1024];
    for (int b = threadIdx.x; b < 1024; b += kBlock) hist[b] = 0u;
    __syncthreads();
    const Chunk c = my_chunk(g.n);
    constexpr int kMatchShift = LEVEL == 2 ? 20 : 10;
    const uint32_t want = sel->prefix >> kMatchShift;
    if (c.base < g.n) {
        float p[kSteps];
        load_sel<FROM_STATE>(g, st, c, p);
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            uint32_t key = key_of(p[j]);
            bool valid = c.full || c.base + 64 * j + c.lane < g.n;
            if (valid && (key >> kMatchShift) == want) atomicAdd(&hist[(key >> (kMatchShift - 10)) & 1023u], 1u);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < 1024; b += kBlock) {
        uint32_t h = hist[b];
        if (h) atomicAdd(&ghist[b], h);
    }
}

// ---------------------------------------------------------------------------
// per tile: keys above / equal to the threshold
// ---------------------------------------------------------------------------
template <bool FROM_STATE>
__global__ __launch_bounds__(kBlock) void sparse_count_k(GroupView g, const float *st, const SelectState *sel,
                                                         uint32_t *tile_gt, uint32_t *tile_eq)
{
    __shared__ uint32_t wgt[kWavesPerBlock], weq[kWavesPerBlock];
    const Chunk c = my_chunk(g.n);
    const uint32_t T = sel->prefix;
    uint32_t ngt = 0, neq = 0;
    if (c.base < g.n) {
        float p[kSteps];
        load_sel<FROM_STATE>(g, st, c, p);
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            uint32_t key = key_of(p[j]);
            bool valid = c.full || c.base + 64 * j + c.lane < g.n;
            ngt += __popcll(__builtin_amdgcn_ballot_w64(valid && key > T));
            neq += __popcll(__builtin_amdgcn_ballot_w64(valid && key == T));
        }
    }
    if (c.lane == 0) { wgt[threadIdx.x >> 6] = ngt; weq[threadIdx.x >> 6] = neq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        tile_gt[blockIdx.x] = wgt[0] + wgt[1] + wgt[2] + wgt[3];
        tile_eq[blockIdx.x] = weq[0] + weq[1] + weq[2] + weq[3];
    }
}

// ---------------------------------------------------------------------------
// one block: exclusive prefix sums of the per-tile counts, in place
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void sparse_scan_k(uint32_t *tile_gt, uint32_t *tile_eq, uint32_t ntiles)
{
    __shared__ uint32_t sg[kBlock], se[kBlock];
    const uint32_t t = threadIdx.x;
    const uint32_t per = (ntiles + kBlock - 1) / kBlock;
    const uint32_t lo = t * per < ntiles ? t * per : ntiles;
    const uint32_t hi = lo + per < ntiles ? lo + per : ntiles;
    uint32_t ag = 0, ae = 0;
    for (uint32_t i = lo; i < hi; ++i) { ag += tile_gt[i]; ae += tile_eq[i]; }
    sg[t] = ag; se[t] = ae;
    __syncthreads();
    for (int d = 1; d < kBlock; d <<= 1) {
        uint32_t xg = t >= (uint32_t)d ? sg[t - d] : 0u, xe = t >= (uint32_t)d ? se[t - d] : 0u;
        __syncthreads();
        sg[t] += xg; se[t] += xe;
        __syncthreads();
    }
    uint32_t rg = sg[t] - ag, re = se[t] - ae;      // exclusive offsets of this thread's run
    for (uint32_t i = lo; i < hi; ++i) {
        uint32_t cg = tile_gt[i], ce = tile_eq[i];
        tile_gt[i] = rg; tile_eq[i] = re;
        rg += cg; re += ce;
    }
}

// ---------------------------------------------------------------------------
// ordered compaction.  An element is kept if its key is above the threshold, or
// equal to it and among the first `need` equal keys in index order.  Its slot
// is (#kept before it) = (#above before it) + min(#equal before it, need).
// ---------------------------------------------------------------------------
template <int ALGO, bool EF, bool FROM_STATE>
__global__ __launch_bounds__(kBlock) void sparse_emit_k(GroupView g, float *st, const SelectState *sel,
                                                        const uint32_t *tile_gt, const uint32_t *tile_eq,
                                                        PayloadHeader *hdr, uint64_t k)
{
    __shared__ uint32_t wgt[kWavesPerBlock], weq[kWavesPerBlock];
    const Chunk c = my_chunk(g.n);
    const uint32_t T = sel->prefix;
    const uint64_t need = sel->need;
    uint32_t *idx = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(hdr) + kHeaderBytes);
    float *val = reinterpret_cast<float *>(idx + k);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        PayloadHeader h;
        h.magic = kMagic; h.algo = ALGO; h.n = g.n; h.k = k; h.scale = 0.0f; h.levels = 0;
        for (int i = 0; i < 8; ++i) h.pad[i] = 0;
        *hdr = h;
    }
    float p[kSteps];
    uint64_t bgt[kSteps], beq[kSteps];
    uint32_t ngt = 0, neq = 0;
    const bool active = c.base < g.n;
    if (active) {
        load_sel<FROM_STATE>(g, st, c, p);
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            uint32_t key = key_of(p[j]);
            bool valid = c.full || c.base + 64 * j + c.lane < g.n;
            bgt[j] = __builtin_amdgcn_ballot_w64(valid && key > T);
            beq[j] = __builtin_amdgcn_ballot_w64(valid && key == T);
            ngt += __popcll(bgt[j]);
            neq += __popcll(beq[j]);
        }
    }
    const uint32_t wave = threadIdx.x >> 6;
    if (c.lane == 0) { wgt[wave] = ngt; weq[wave] = neq; }
    __syncthreads();
    if (!active) return;
    uint64_t gt_before = tile_gt[blockIdx.x], eq_before = tile_eq[blockIdx.x];
    for (uint32_t w = 0; w < wave; ++w) { gt_before += wgt[w]; eq_before += weq[w]; }
    const uint64_t lane_bit = 1ull << c.lane;
#pragma unroll
    for (int j = 0; j < kSteps; ++j) {
        uint64_t gtb = gt_before + lanes_below(bgt[j]);
        uint64_t eqb = eq_before + lanes_below(beq[j]);
        bool is_gt = (bgt[j] & lane_bit) != 0, is_eq = (beq[j] & lane_bit) != 0;
        if (is_gt || (is_eq && eqb < need)) {
            uint64_t pos = gtb + (eqb < need ? eqb : need);
            uint32_t i = c.base + 64 * j + c.lane;
            if (pos < k) {                       // always true for a consistent threshold; guards the payload bounds
                idx[pos] = i;
                val[pos] = p[j];
            }
            if (ALGO == MC_ALGO_DGC) { st[i] = 0.0f; st[(size_t)g.n + i] = 0.0f; }   // momentum factor masking
            else if (EF) st[i] = 0.0f;
        }
        gt_before += __popcll(bgt[j]);
        eq_before += __popcll(beq[j]);
    }
}

template <int ALGO, bool EF>
static void sparse_compress_t(const LaunchCtx &lc, const GroupView &g, float *st, float momentum, uint64_t k,
                              PayloadHeader *hdr, const SparseScratch &sc)
{
    constexpr bool FS = (ALGO == MC_ALGO_DGC) || EF;
    const uint32_t nt = tiles_of(g.n);
    dim3 grid(nt), block(kBlock), one(1);
    uint32_t *h1 = sc.hist, *h2 = sc.hist + kBins1, *h3 = sc.hist + kBins1 + kBins2;
    prof_begin(lc, K_SPARSE_ACCUM);
    hipLaunchKernelGGL((sparse_accum_k<ALGO, EF>), grid, block, 0, lc.stream, g, st, momentum, h1);
    prof_end(lc, K_SPARSE_ACCUM);
    prof_begin(lc, K_SELECT_BIN);
    hipLaunchKernelGGL(select_bin_k<kBins1>, one, block, 0, lc.stream, h1, sc.sel, 1, k, 20);
    prof_end(lc, K_SELECT_BIN);
    prof_begin(lc, K_SPARSE_HIST);
    hipLaunchKernelGGL((sparse_hist_k<FS, 2>), grid, block, 0, lc.stream, g, st, sc.sel, h2);
    prof_end(lc, K_SPARSE_HIST);
    prof_begin(lc, K_SELECT_BIN);
    hipLaunchKernelGGL(select_bin_k<kBins2>, one, block, 0, lc.stream, h2, sc.sel, 0, k, 10);
    prof_end(lc, K_SELECT_BIN);
    prof_begin(lc, K_SPARSE_HIST);
    hipLaunchKernelGGL((sparse_hist_k<FS, 3>), grid, block, 0, lc.stream, g, st, sc.sel, h3);
    prof_end(lc, K_SPARSE_HIST);
    prof_begin(lc, K_SELECT_BIN);
    hipLaunchKernelGGL(select_bin_k<kBins3>, one, block, 0, lc.stream, h3, sc.sel, 0, k, 0);
    prof_end(lc, K_SELECT_BIN);
    prof_begin(lc, K_SPARSE_COUNT);
    hipLaunchKernelGGL(sparse_count_k<FS>, grid, block, 0, lc.stream, g, st, sc.sel, sc.tile_gt, sc.tile_eq);
    prof_end(lc, K_SPARSE_COUNT);
    prof_begin(lc, K_SPARSE_SCAN);
    hipLaunchKernelGGL(sparse_scan_k, one, block, 0, lc.stream, sc.tile_gt, sc.tile_eq, nt);
    prof_end(lc, K_SPARSE_SCAN);
    prof_begin(lc, K_SPARSE_EMIT);
    hipLaunchKernelGGL((sparse_emit_k<ALGO, EF, FS>), grid, block, 0, lc.stream, g, st, sc.sel, sc.tile_gt, sc.tile_eq, hdr, k);
    prof_end(lc, K_SPARSE_EMIT);
}

void launch_sparse_compress(const LaunchCtx &lc, int algo, const GroupView &g, bool ef, float *state_f, float momentum,
                            uint64_t k, PayloadHeader *hdr, const SparseScratch &sc)
{
    if (g.n == 0) return;
    if (algo == MC_ALGO_DGC) sparse_compress_t<MC_ALGO_DGC, true>(lc, g, state_f, momentum, k, hdr, sc);
    else if (ef) sparse_compress_t<MC_ALGO_TOPK, true>(lc, g, state_f, momentum, k, hdr, sc);
    else sparse_compress_t<MC_ALGO_TOPK, false>(lc, g, state_f, momentum, k, hdr, sc);
}

// ---------------------------------------------------------------------------
// Sparse decompress-and-sum.  Every worker's indices ascend, so a 4096-element
// output tile owns one contiguous run of each list (found by binary search).
// The tile is accumulated in LDS, one worker after the other in ascending worker
// order -- the same order of fp32 additions as a dense sum, since adding the +0
// of an absent entry changes nothing -- and written once.  No atomics, no
// pre-zeroed output, bit-reproducible.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lower_bound_u32(const uint32_t *a, uint32_t k, uint32_t x)
{
    uint32_t lo = 0, hi = k;
    while (lo < hi) {
        uint32_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(kBlock) void sparse_decompress_k(int algo, GroupView out, PayloadPtrs pl, int W, float alpha,
                                                              uint64_t k64, int *status)
{
    __shared__ float acc[kTile];
    __shared__ uint32_t lo_s[kMaxWorkers], hi_s[kMaxWorkers];
    const uint32_t k = (uint32_t)k64;
    const uint32_t tb = blockIdx.x * (uint32_t)kTile;
    const uint32_t t = threadIdx.x;
    if (blockIdx.x == 0 && (int)t < W) {
        const PayloadHeader *h = reinterpret_cast<const PayloadHeader *>(pl.p[t]);
        if (h->magic != kMagic || h->algo != (uint32_t)algo || h->n != (uint64_t)out.n || h->k != k64) *status = 1;
    }
#pragma unroll
    for (int j = 0; j < kSteps; ++j) acc[t + kBlock * j] = 0.0f;
    if ((int)t < 2 * W) {
        int w = t < (uint32_t)W ? t : t - W;
        const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w] + kHeaderBytes);
        // the tile end saturates: tb + kTile may exceed n but not 2^32 (n < 2^32 - 2^24)
        uint32_t r = lower_bound_u32(idx, k, t < (uint32_t)W ? tb : tb + (uint32_t)kTile);
        if (t < (uint32_t)W) lo_s[w] = r; else hi_s[w] = r;
    }
    __syncthreads();
    for (int w = 0; w < W; ++w) {
        const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w] + kHeaderBytes);
        const float *val = reinterpret_cast<const float *>(idx + k);
        const uint32_t hi = hi_s[w];
        for (uint32_t e = lo_s[w] + t; e < hi; e += kBlock) {
            uint32_t local = idx[e] - tb;
            if (local < (uint32_t)kTile) acc[local] = acc[local] + val[e];
        }
        __syncthreads();
    }
    const Chunk c = my_chunk(out.n);
    if (c.base >= out.n) return;
    float v[kSteps];
    const float *mine = acc + (c.base - tb) + c.lane;
#pragma unroll
    for (int j = 0; j < kSteps; ++j) v[j] = alpha * mine[64 * j];
    store_seg(out, c, v);
}

void launch_sparse_decompress(const LaunchCtx &lc, int algo, const GroupView &out, const PayloadPtrs &pl, int W,
                              float alpha, uint64_t k, int *status)
{
    if (out.n == 0) return;
    prof_begin(lc, K_SPARSE_DECOMPRESS);
    hipLaunchKernelGGL(sparse_decompress_k, dim3(tiles_of(out.n)), dim3(kBlock), 0, lc.stream, algo, out, pl, W, alpha, k, status);
    prof_end(lc, K_SPARSE_DECOMPRESS);
}

}  // namespace mc
