// Sparsifiers (Top-k, DGC) for gfx950: exact top-k of |p| over a whole merged
// group, ties at the threshold taken in index order (lower index wins), payload
// written in ascending index order, and the sparse decompress-and-sum.
//
// The paper singles out the top-k() operation as the cost that merging alone
// does not remove (Section 5.1).  Here the selection is a radix select on the
// 31-bit magnitude key (11 + 10 + 10 bits) that never sorts and, in the steady
// state, touches the gradient once:
//
//   accumulate   p = g + e (DGC: u = m u + g, v = v + u) streamed once; every element
//                whose key reaches a *hint* (a little below the last threshold of this
//                group) is copied, in index order, into the candidate slots of its
//                1024-element chunk, and counted in the level-1 histogram
//   refill       runs only if fewer than k candidates were found (first call, or the
//                distribution moved): makes every element a candidate
//   hist 2, 3    each block first resolves the previous level from its histogram,
//                then histograms the candidates that match the prefix
//   count        resolves level 3 (threshold key T, number of keys == T to take),
//                counts kept candidates per block / wavefront, publishes the next hint
//   emit         ordered compaction of the kept candidates into (idx, val); kept
//                entries leave the residual
//
// If at least k elements have key >= hint, the k-th largest key T is >= hint, so
// every element with key >= T is a candidate and the result is exact whatever the
// hint was; the hint only decides how much work the later kernels have.
// No kernel waits on another block: every dependency is a kernel boundary.
#include "mc_internal.h"

namespace mc {

static inline uint32_t tiles_of(uint32_t n) { return (uint32_t)(((uint64_t)n + kTile - 1) / kTile); }
static inline uint32_t chunks_of(uint32_t n) { return (uint32_t)(((uint64_t)n + kChunk - 1) / kChunk); }

constexpr int kBins1 = 2048, kBins2 = 1024, kBins3 = 1024;
constexpr uint32_t kHintMargin = 3u << 19;   // 3/16 of an octave below the last threshold

__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

__device__ __forceinline__ Chunk chunk_at(uint32_t tile, uint32_t n)
{
    Chunk c;
    uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.base = tile * (uint32_t)kTile + wave * (uint32_t)kChunk;
    c.lane = threadIdx.x & 63u;
    c.full = c.base < n && n - c.base >= (uint32_t)kChunk;
    return c;
}

__device__ __forceinline__ void flush_hist(const uint32_t *lds, uint32_t *global, int bins)
{
    for (int b = threadIdx.x; b < bins; b += kBlock) {
        uint32_t h = lds[b];
        if (h) atomicAdd(&global[b], h);
    }
}

// Copy the flagged elements of a chunk, in index order, into the chunk's candidate slots.
__device__ __forceinline__ uint32_t put_candidates(const Chunk &c, const float (&p)[kSteps], const uint64_t (&flag)[kSteps],
                                                   uint32_t *cand_bits, uint16_t *cand_loc, uint32_t *hist /* LDS */)
{
    uint32_t run = 0;
    const uint64_t me = 1ull << c.lane;
#pragma unroll
    for (int j = 0; j < kSteps; ++j) {
        if (flag[j] & me) {
            uint32_t slot = c.base + run + lanes_below(flag[j]);
            cand_bits[slot] = __float_as_uint(p[j]);
            cand_loc[slot] = (uint16_t)(64 * j + c.lane);
            atomicAdd(&hist[key_of(p[j]) >> 20], 1u);
        }
        run += __popcll(flag[j]);
    }
    return run;
}

// ---------------------------------------------------------------------------
// accumulate + candidate filter + level-1 histogram of the candidates
// ---------------------------------------------------------------------------
template <int ALGO, bool EF>
__global__ __launch_bounds__(kBlock) void sparse_accum_k(GroupView g, float *st, float momentum, SparseScratch sc)
{
    __shared__ uint32_t hist[kBins1];
    __shared__ uint32_t wcnt[kWavesPerBlock];
    for (int b = threadIdx.x; b < kBins1; b += kBlock) hist[b] = 0u;
    __syncthreads();
    const Chunk c = my_chunk(g.n);
    const uint32_t hint = *sc.hint;
    uint32_t run = 0;
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
        uint64_t flag[kSteps];
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            bool valid = c.full || c.base + 64 * j + c.lane < g.n;
            flag[j] = __builtin_amdgcn_ballot_w64(valid && key_of(p[j]) >= hint);
        }
        run = put_candidates(c, p, flag, sc.cand_bits, sc.cand_loc, hist);
        if (c.lane == 0) sc.run[c.base >> 10] = run;
    }
    if (c.lane == 0) wcnt[threadIdx.x >> 6] = run;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
        if (t) atomicAdd(sc.total, (unsigned long long)t);
    }
    flush_hist(hist, sc.hist, kBins1);
}

// the vector the selection works on: v / p kept in the state, or the gradient itself
template <bool FROM_STATE>
__device__ __forceinline__ void load_sel(const GroupView &g, const float *st, const Chunk &c, float (&p)[kSteps])
{
    if (FROM_STATE) load_flat(st, c, g.n, p, 0.0f);
    else load_seg(g, c, p);
}

// ---------------------------------------------------------------------------
// refill: only if the hint left fewer than k candidates.  Every element becomes a
// candidate; the elements below the hint (not counted yet) join the histogram.
// ---------------------------------------------------------------------------
template <bool FROM_STATE>
__global__ __launch_bounds__(kBlock) void sparse_refill_k(GroupView g, const float *st, uint64_t k, SparseScratch sc)
{
    __shared__ uint32_t hist[kBins1];
    if (*sc.total >= k) return;
    for (int b = threadIdx.x; b < kBins1; b += kBlock) hist[b] = 0u;
    __syncthreads();
    const uint32_t hint = *sc.hint;
    const uint32_t ntiles = (g.n + (uint32_t)kTile - 1u) / (uint32_t)kTile;
    for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const Chunk c = chunk_at(tile, g.n);
        if (c.base >= g.n) continue;
        float p[kSteps];
        load_sel<FROM_STATE>(g, st, c, p);
        uint32_t cnt = 0;
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            uint32_t i = c.base + 64 * j + c.lane;
            if (c.full || i < g.n) {
                sc.cand_bits[i] = __float_as_uint(p[j]);
                sc.cand_loc[i] = (uint16_t)(64 * j + c.lane);
                if (key_of(p[j]) < hint) atomicAdd(&hist[key_of(p[j]) >> 20], 1u);
                cnt = 64 * j + c.lane + 1;
            }
        }
        // elements of the chunk = largest valid local index + 1, held by the last valid lane
        uint32_t m = cnt;
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) { uint32_t o = __shfl_xor(m, s, 64); m = o > m ? o : m; }
        if (c.lane == 0) sc.run[c.base >> 10] = m;
    }
    __syncthreads();
    flush_hist(hist, sc.hist, kBins1);
}

// ---------------------------------------------------------------------------
// Resolve one radix level, by every thread block for itself: find the bin b with
//   count(bins > b) < need <= count(bins >= b)
// Returns through LDS: out[0] = bin, out[1..2] = need - count(bins > b) (lo, hi).
// ---------------------------------------------------------------------------
template <int BINS>
__device__ __forceinline__ void resolve_level(const uint32_t *ghist, uint64_t need, uint64_t *above /* kBlock */,
                                              uint32_t *out /* 3 */)
{
    constexpr int kPer = BINS / kBlock;
    const int t = threadIdx.x;
    uint32_t h[kPer];
    uint64_t own = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) { h[i] = ghist[t * kPer + i]; own += h[i]; }
    if (t == 0) { out[0] = 0u; out[1] = 0u; out[2] = 0u; }    // defined result even for an inconsistent histogram
    above[t] = own;
    __syncthreads();
    for (int d = 1; d < kBlock; d <<= 1) {               // inclusive suffix sum over threads
        uint64_t add = t + d < kBlock ? above[t + d] : 0;
        __syncthreads();
        above[t] += add;
        __syncthreads();
    }
    uint64_t run = above[t] - own;                        // keys in bins owned by higher threads
    if (run < need && need <= run + own) {
#pragma unroll
        for (int i = kPer - 1; i >= 0; --i) {
            if (run < need && need <= run + h[i]) {
                uint64_t rest = need - run;
                out[0] = (uint32_t)(t * kPer + i);
                out[1] = (uint32_t)rest;
                out[2] = (uint32_t)(rest >> 32);
            }
            run += h[i];
        }
    }
    __syncthreads();
}

// chunks [first, last) owned by a block of the candidate kernels, and by each of its wavefronts
struct ChunkRange { uint32_t first, last; };
__device__ __forceinline__ ChunkRange wave_range(uint32_t nchunks, uint32_t per_wave)
{
    uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint64_t first = ((uint64_t)blockIdx.x * kWavesPerBlock + wave) * per_wave;
    ChunkRange r;
    r.first = first < nchunks ? (uint32_t)first : nchunks;
    r.last = first + per_wave < nchunks ? (uint32_t)(first + per_wave) : nchunks;
    return r;
}

// ---------------------------------------------------------------------------
// level 2 / level 3 histogram over the candidates
//   LEVEL 2: resolves level 1 (2048 bins, need = k), histograms bits 19..10 of matching keys
//   LEVEL 3: resolves level 2 (1024 bins), histograms bits 9..0
// Block 0 records the resolved prefix for the next kernel and clears the histogram
// that the previous kernel has finished reading.
// ---------------------------------------------------------------------------
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void cand_hist_k(uint32_t nchunks, uint32_t per_wave, uint64_t k, SparseScratch sc)
{
    __shared__ uint32_t hist[1024];
    __shared__ uint64_t above[kBlock];
    __shared__ uint32_t res[3];
    for (int b = threadIdx.x; b < 1024; b += kBlock) hist[b] = 0u;
    uint32_t *h1 = sc.hist, *h2 = sc.hist + kBins1, *h3 = h2 + kBins2;
    uint32_t prefix;
    if (LEVEL == 2) {
        resolve_level<kBins1>(h1, k, above, res);
        prefix = res[0] << 20;
    } else {
        const SelectState s1 = sc.sel[1];
        resolve_level<kBins2>(h2, s1.need, above, res);
        prefix = s1.prefix | (res[0] << 10);
    }
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            SelectState s;
            s.prefix = prefix; s.pad0 = 0; s.need = (uint64_t)res[1] | ((uint64_t)res[2] << 32);
            sc.sel[LEVEL == 2 ? 1 : 2] = s;
        }
        if (LEVEL == 3) for (int b = threadIdx.x; b < kBins1; b += kBlock) h1[b] = 0u;   // level 2 is done with it
    }
    constexpr int kMatchShift = LEVEL == 2 ? 20 : 10;
    const uint32_t want = prefix >> kMatchShift;
    const ChunkRange r = wave_range(nchunks, per_wave);
    const uint32_t lane = threadIdx.x & 63u;
    for (uint32_t ch = r.first; ch < r.last; ++ch) {
        const uint32_t cnt = sc.run[ch];
        const uint32_t *bits = sc.cand_bits + (size_t)ch * kChunk;
        for (uint32_t e = lane; e < cnt; e += 64) {
            uint32_t key = bits[e] & 0x7FFFFFFFu;
            if ((key >> kMatchShift) == want) atomicAdd(&hist[(key >> (kMatchShift - 10)) & 1023u], 1u);
        }
    }
    __syncthreads();
    flush_hist(hist, LEVEL == 2 ? h2 : h3, 1024);
}

// ---------------------------------------------------------------------------
// count: resolve level 3 -> threshold key T and `need` (keys == T to take, in
// index order); kept candidates per wavefront and per block.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void cand_count_k(uint32_t nchunks, uint32_t per_wave, SparseScratch sc)
{
    __shared__ uint64_t above[kBlock];
    __shared__ uint32_t res[3];
    __shared__ uint32_t wgt[kWavesPerBlock], weq[kWavesPerBlock];
    const SelectState s2 = sc.sel[2];
    resolve_level<kBins3>(sc.hist + kBins1 + kBins2, s2.need, above, res);
    const uint32_t T = s2.prefix | res[0];
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            SelectState s;
            s.prefix = T; s.pad0 = 0; s.need = (uint64_t)res[1] | ((uint64_t)res[2] << 32);
            sc.sel[3] = s;
            *sc.hint = T > kHintMargin ? T - kHintMargin : 0u;      // where the next call starts filtering
        }
        for (int b = threadIdx.x; b < kBins2; b += kBlock) sc.hist[kBins1 + b] = 0u;      // level 3 is done with it
    }
    const ChunkRange r = wave_range(nchunks, per_wave);
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t ngt = 0, neq = 0;
    for (uint32_t ch = r.first; ch < r.last; ++ch) {
        const uint32_t cnt = sc.run[ch];
        const uint32_t *bits = sc.cand_bits + (size_t)ch * kChunk;
        for (uint32_t e0 = 0; e0 < cnt; e0 += 64) {
            uint32_t e = e0 + lane;
            uint32_t key = e < cnt ? bits[e] & 0x7FFFFFFFu : 0u;
            ngt += __popcll(__builtin_amdgcn_ballot_w64(e < cnt && key > T));
            neq += __popcll(__builtin_amdgcn_ballot_w64(e < cnt && key == T));
        }
    }
    const uint32_t wave = threadIdx.x >> 6;
    if (lane == 0) {
        wgt[wave] = ngt; weq[wave] = neq;
        sc.wave_gt[blockIdx.x * kWavesPerBlock + wave] = ngt;
        sc.wave_eq[blockIdx.x * kWavesPerBlock + wave] = neq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        sc.blk_gt[blockIdx.x] = wgt[0] + wgt[1] + wgt[2] + wgt[3];
        sc.blk_eq[blockIdx.x] = weq[0] + weq[1] + weq[2] + weq[3];
    }
}

// ---------------------------------------------------------------------------
// emit: ordered compaction.  A candidate is kept if its key is above T, or equal
// to T and among the first `need` such keys in index order.  Its slot is
//   (#kept before it) = (#above before it) + min(#equal before it, need).
// Every block adds up the counts of the blocks before it; nothing waits.
// ---------------------------------------------------------------------------
template <int ALGO, bool EF>
__global__ __launch_bounds__(kBlock) void cand_emit_k(uint32_t n, uint32_t nchunks, uint32_t per_wave, float *st,
                                                      PayloadHeader *hdr, uint64_t k, SparseScratch sc)
{
    __shared__ uint64_t sgt[kBlock], seq[kBlock];
    const SelectState s3 = sc.sel[3];
    const uint32_t T = s3.prefix;
    const uint64_t need = s3.need;
    uint32_t *idx = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(hdr) + kHeaderBytes);
    float *val = reinterpret_cast<float *>(idx + k);
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            PayloadHeader h;
            h.magic = kMagic; h.algo = ALGO; h.n = n; h.k = k; h.scale = 0.0f; h.levels = 0;
            for (int i = 0; i < 8; ++i) h.pad[i] = 0;
            *hdr = h;
            *sc.total = 0ull;
        }
        for (int b = threadIdx.x; b < kBins3; b += kBlock) sc.hist[kBins1 + kBins2 + b] = 0u;   // count is done with it
    }
    // kept-before of this block: sum over the blocks before it
    uint64_t ag = 0, ae = 0;
    for (uint32_t b = threadIdx.x; b < blockIdx.x; b += kBlock) { ag += sc.blk_gt[b]; ae += sc.blk_eq[b]; }
    sgt[threadIdx.x] = ag; seq[threadIdx.x] = ae;
    __syncthreads();
    for (int s = kBlock / 2; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) { sgt[threadIdx.x] += sgt[threadIdx.x + s]; seq[threadIdx.x] += seq[threadIdx.x + s]; }
        __syncthreads();
    }
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint64_t gt_before = sgt[0], eq_before = seq[0];
    for (uint32_t w = 0; w < wave; ++w) {
        gt_before += sc.wave_gt[blockIdx.x * kWavesPerBlock + w];
        eq_before += sc.wave_eq[blockIdx.x * kWavesPerBlock + w];
    }
    const ChunkRange r = wave_range(nchunks, per_wave);
    const uint32_t lane = threadIdx.x & 63u;
    for (uint32_t ch = r.first; ch < r.last; ++ch) {
        const uint32_t cnt = sc.run[ch];
        const uint32_t *bits = sc.cand_bits + (size_t)ch * kChunk;
        const uint16_t *loc = sc.cand_loc + (size_t)ch * kChunk;
        for (uint32_t e0 = 0; e0 < cnt; e0 += 64) {
            uint32_t e = e0 + lane;
            uint32_t b = e < cnt ? bits[e] : 0u;
            uint32_t key = b & 0x7FFFFFFFu;
            bool is_gt = e < cnt && key > T, is_eq = e < cnt && key == T;
            uint64_t bgt = __builtin_amdgcn_ballot_w64(is_gt), beq = __builtin_amdgcn_ballot_w64(is_eq);
            uint64_t gtb = gt_before + lanes_below(bgt), eqb = eq_before + lanes_below(beq);
            if (is_gt || (is_eq && eqb < need)) {
                uint64_t pos = gtb + (eqb < need ? eqb : need);
                uint32_t i = ch * (uint32_t)kChunk + loc[e];
                if (pos < k && i < n) {                  // always true for consistent scratch; guards the buffers
                    idx[pos] = i;
                    val[pos] = __uint_as_float(b);
                    if (ALGO == MC_ALGO_DGC) { st[i] = 0.0f; st[(size_t)n + i] = 0.0f; }   // momentum factor masking
                    else if (EF) st[i] = 0.0f;
                }
            }
            gt_before += __popcll(bgt);
            eq_before += __popcll(beq);
        }
    }
}

// geometry of the candidate kernels: at most 1024 blocks, each wavefront a contiguous run of chunks
static inline void cand_geometry(uint32_t nchunks, uint32_t *blocks, uint32_t *per_wave)
{
    const uint32_t max_waves = kMaxCandBlocks * kWavesPerBlock;
    uint32_t pw = (nchunks + max_waves - 1) / max_waves;
    if (pw < 1) pw = 1;
    uint32_t waves = (nchunks + pw - 1) / pw;
    *per_wave = pw;
    *blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
    if (*blocks < 1) *blocks = 1;
}

template <int ALGO, bool EF>
static void sparse_compress_t(const LaunchCtx &lc, const GroupView &g, float *st, float momentum, uint64_t k,
                              PayloadHeader *hdr, const SparseScratch &sc)
{
    constexpr bool FS = (ALGO == MC_ALGO_DGC) || EF;
    const uint32_t nt = tiles_of(g.n), nch = chunks_of(g.n);
    uint32_t cblocks, per_wave;
    cand_geometry(nch, &cblocks, &per_wave);
    dim3 grid(nt), block(kBlock), cgrid(cblocks), rgrid(nt < 1024 ? nt : 1024);
    prof_begin(lc, K_SPARSE_ACCUM);
    hipLaunchKernelGGL((sparse_accum_k<ALGO, EF>), grid, block, 0, lc.stream, g, st, momentum, sc);
    prof_end(lc, K_SPARSE_ACCUM);
    prof_begin(lc, K_SPARSE_REFILL);
    hipLaunchKernelGGL(sparse_refill_k<FS>, rgrid, block, 0, lc.stream, g, st, k, sc);
    prof_end(lc, K_SPARSE_REFILL);
    prof_begin(lc, K_CAND_HIST);
    hipLaunchKernelGGL(cand_hist_k<2>, cgrid, block, 0, lc.stream, nch, per_wave, k, sc);
    prof_end(lc, K_CAND_HIST);
    prof_begin(lc, K_CAND_HIST);
    hipLaunchKernelGGL(cand_hist_k<3>, cgrid, block, 0, lc.stream, nch, per_wave, k, sc);
    prof_end(lc, K_CAND_HIST);
    prof_begin(lc, K_CAND_COUNT);
    hipLaunchKernelGGL(cand_count_k, cgrid, block, 0, lc.stream, nch, per_wave, sc);
    prof_end(lc, K_CAND_COUNT);
    prof_begin(lc, K_CAND_EMIT);
    hipLaunchKernelGGL((cand_emit_k<ALGO, EF>), cgrid, block, 0, lc.stream, g.n, nch, per_wave, st, hdr, k, sc);
    prof_end(lc, K_CAND_EMIT);
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
// output tile owns one contiguous run of each list.  A first kernel writes, per
// worker, where each tile's run starts (one thread per payload entry, no search);
// the second accumulates each tile in LDS, one worker after the other in ascending
// worker order -- the same order of fp32 additions as a dense sum, since adding
// the +0 of an absent entry changes nothing -- and writes it once.  No atomics, no
// pre-zeroed output, bit-reproducible.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void sparse_index_k(int algo, uint32_t n, PayloadPtrs pl, int W, uint64_t k64,
                                                         uint32_t ntiles, uint32_t *tile_off, int *status)
{
    const uint32_t k = (uint32_t)k64;
    const uint32_t w = blockIdx.y;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const PayloadHeader *h = reinterpret_cast<const PayloadHeader *>(pl.p[w]);
        if (h->magic != kMagic || h->algo != (uint32_t)algo || h->n != (uint64_t)n || h->k != k64) *status = 1;
    }
    const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w] + kHeaderBytes);
    uint32_t *off = tile_off + (size_t)w * (ntiles + 1);
    const uint32_t e = blockIdx.x * kBlock + threadIdx.x;
    if (e > k) return;
    // entry e starts the runs of all tiles after the tile of entry e-1, up to and including its own;
    // the virtual entry k (one past the end) closes the tiles behind the last entry
    int64_t t_prev = e == 0 ? -1 : (int64_t)(idx[e - 1] >> 12);
    int64_t t_cur = e == k ? (int64_t)ntiles : (int64_t)(idx[e] >> 12);
    if (t_cur > (int64_t)ntiles) t_cur = ntiles;
    for (int64_t t = t_prev + 1; t <= t_cur; ++t) off[t] = e;
}

constexpr int kSparseBatch = 8;

__global__ __launch_bounds__(kBlock) void sparse_decompress_k(GroupView out, PayloadPtrs pl, int W, float alpha,
                                                              uint64_t k64, uint32_t ntiles, const uint32_t *tile_off)
{
    __shared__ float acc[kTile];
    const uint32_t k = (uint32_t)k64;
    const uint32_t tb = blockIdx.x * (uint32_t)kTile;
    const uint32_t t = threadIdx.x;
#pragma unroll
    for (int j = 0; j < kSteps; ++j) acc[t + kBlock * j] = 0.0f;
    __syncthreads();
    for (int w0 = 0; w0 < W; w0 += kSparseBatch) {
        // issue the loads of a batch of workers before the first LDS update
        uint32_t lo[kSparseBatch], hi[kSparseBatch];
#pragma unroll
        for (int b = 0; b < kSparseBatch; ++b) {
            lo[b] = hi[b] = 0;
            if (w0 + b < W) {
                const uint32_t *off = tile_off + (size_t)(w0 + b) * (ntiles + 1) + blockIdx.x;
                lo[b] = off[0]; hi[b] = off[1];
                lo[b] = lo[b] < k ? lo[b] : k;
                hi[b] = hi[b] < k ? hi[b] : k;
                if (hi[b] - lo[b] > (uint32_t)kTile) hi[b] = lo[b];      // inconsistent payload: a tile holds at most 4096
            }
        }
        uint32_t ix[kSparseBatch];
        float vv[kSparseBatch];
#pragma unroll
        for (int b = 0; b < kSparseBatch; ++b) {
            ix[b] = 0xFFFFFFFFu; vv[b] = 0.0f;
            if (w0 + b < W && lo[b] + t < hi[b]) {
                const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w0 + b] + kHeaderBytes);
                ix[b] = ld_stream(idx + lo[b] + t);
                vv[b] = ld_stream(reinterpret_cast<const float *>(idx + k) + lo[b] + t);
            }
        }
#pragma unroll
        for (int b = 0; b < kSparseBatch; ++b) {
            if (w0 + b < W) {
                uint32_t local = ix[b] - tb;
                if (ix[b] != 0xFFFFFFFFu && local < (uint32_t)kTile) acc[local] = acc[local] + vv[b];
                // the rare tile with more than 256 entries of one worker
                const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w0 + b] + kHeaderBytes);
                const float *val = reinterpret_cast<const float *>(idx + k);
                for (uint32_t e = lo[b] + kBlock + t; e < hi[b]; e += kBlock) {
                    uint32_t l2 = idx[e] - tb;
                    if (l2 < (uint32_t)kTile) acc[l2] = acc[l2] + val[e];
                }
                __syncthreads();
            }
        }
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
                              float alpha, uint64_t k, uint32_t *tile_off, int *status)
{
    if (out.n == 0) return;
    const uint32_t nt = tiles_of(out.n);
    prof_begin(lc, K_SPARSE_INDEX);
    hipLaunchKernelGGL(sparse_index_k, dim3((uint32_t)((k + 1 + kBlock - 1) / kBlock), W), dim3(kBlock), 0, lc.stream, algo,
                       out.n, pl, W, k, nt, tile_off, status);
    prof_end(lc, K_SPARSE_INDEX);
    prof_begin(lc, K_SPARSE_DECOMPRESS);
    hipLaunchKernelGGL(sparse_decompress_k, dim3(nt), dim3(kBlock), 0, lc.stream, out, pl, W, alpha, k, nt, tile_off);
    prof_end(lc, K_SPARSE_DECOMPRESS);
}

}  // namespace mc
