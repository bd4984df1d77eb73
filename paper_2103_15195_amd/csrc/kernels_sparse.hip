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
//   plan         one block: lists the non-empty chunks, cuts the candidate sequence into
//                equal shares (one per wavefront of the later kernels; a few tensors hold
//                most candidates), resolves radix level 1.  If fewer than k candidates
//                were found (first call, or the distribution moved) all blocks instead
//                make every element a candidate (refill)
//   hist 2, 3    histogram the candidates that match the prefix resolved so far; the
//                previous level is resolved by every wavefront for itself
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
// Histogram scratch: the three radix levels one after the other.  Global atomics on
// one address serialise (tens of nanoseconds each on this part), so only the bins
// themselves are updated -- no shared summary counters -- and a level is resolved
// by a wavefront that reads all its bins.
constexpr int kHist1 = 0, kHist2 = kHist1 + kBins1, kHist3 = kHist2 + kBins2;
static_assert(kHist3 + kBins3 == kHistWords, "histogram scratch layout");
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

// add a block's LDS histogram to the global one (fine bins only)
__device__ __forceinline__ void flush_fine(const uint32_t *lds, uint32_t *fine, int bins)
{
    for (int b = threadIdx.x; b < bins; b += blockDim.x) {
        uint32_t h = lds[b];
        if (h) atomicAdd(&fine[b], h);
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
        if (ALGO == MC_ALGO_DGC) {
            // momentum correction: u = m u + g ; v = v + u ; the vector compressed is v
            float *vbuf = st, *ubuf = st + g.n;
            float u[kSteps], v[kSteps];
            load_flat(ubuf, c, g.n, u, 0.0f);
            load_flat(vbuf, c, g.n, v, 0.0f);
            load_seg(g, c, p);
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
            load_seg(g, c, p);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) p[j] = p[j] + e[j];
            store_flat(st, c, g.n, p);
        } else {
            load_seg(g, c, p);
        }
        uint64_t flag[kSteps];
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            bool valid = c.full || c.base + 64 * j + c.lane < g.n;
            flag[j] = __builtin_amdgcn_ballot_w64(valid && key_of(p[j]) >= hint);
        }
        run = put_candidates(c, p, flag, sc.cand_bits, sc.cand_loc, hist);
    }
    if (c.lane == 0) wcnt[threadIdx.x >> 6] = run;
    __syncthreads();
    if (threadIdx.x == 0)       // candidates of the tile's four chunks, 16 bits each (a chunk holds at most 1024)
        sc.tile_runs[blockIdx.x] = (uint64_t)wcnt[0] | ((uint64_t)wcnt[1] << 16) | ((uint64_t)wcnt[2] << 32) | ((uint64_t)wcnt[3] << 48);
    flush_fine(hist, sc.hist + kHist1, kBins1);
}

// ---------------------------------------------------------------------------
// Resolve one radix level by a whole block from the fine bins: find the bin b with
//   count(bins > b) < need <= count(bins >= b)        and  rest = need - count(bins > b).
// Result through LDS: out[0] = bin, out[1..2] = rest (lo, hi).  THREADS = blockDim.x.
// ---------------------------------------------------------------------------
template <int BINS, int THREADS>
__device__ __forceinline__ void resolve_block(const uint32_t *fine, uint64_t need, uint64_t *above /* THREADS */,
                                              uint32_t *out /* 3 */)
{
    constexpr int kPer = BINS / THREADS;
    const int t = threadIdx.x;
    uint32_t h[kPer];
    uint64_t own = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) { h[i] = fine[t * kPer + i]; own += h[i]; }
    if (t == 0) { out[0] = 0u; out[1] = 0u; out[2] = 0u; }    // defined result even for an inconsistent histogram
    above[t] = own;
    __syncthreads();
    for (int d = 1; d < THREADS; d <<= 1) {              // inclusive suffix sum over threads
        uint64_t add = t + d < THREADS ? above[t + d] : 0;
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

// ---------------------------------------------------------------------------
// Resolve one radix level inside a wavefront: every lane reads BINS / 64 adjacent
// bins (one vector load), a suffix scan over the lanes finds the lane where the
// running count crosses `need`, and that lane walks its own bins.  One memory
// latency, no block barrier.
// ---------------------------------------------------------------------------
template <int BINS>
__device__ __forceinline__ void resolve_wave(const uint32_t *fine, uint64_t need, uint32_t &bin, uint64_t &rest)
{
    constexpr int kPer = BINS / 64;
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t h[kPer];
    uint64_t own = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) { h[i] = fine[lane * kPer + i]; own += h[i]; }
    uint64_t incl = own;                                    // inclusive suffix sum over lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t o = __shfl_down(incl, d, 64);
        if (lane + d < 64) incl += o;
    }
    uint64_t run = incl - own;                              // keys in the bins of higher lanes
    const bool mine = run < need && need <= incl;
    uint32_t b = 0;
    uint64_t r = 0;
    if (mine) {
#pragma unroll
        for (int i = kPer - 1; i >= 0; --i) {
            if (run < need && need <= run + h[i]) { b = lane * kPer + i; r = need - run; }
            run += h[i];
        }
    }
    const uint64_t hit = __builtin_amdgcn_ballot_w64(mine);
    const uint32_t src = hit ? (uint32_t)__builtin_ctzll(hit) : 0u;     // an inconsistent histogram still gives a defined bin
    bin = __shfl(b, src, 64);
    rest = __shfl(r, src, 64);
}

// the vector the selection works on: v / p kept in the state, or the gradient itself
template <bool FROM_STATE>
__device__ __forceinline__ void load_sel(const GroupView &g, const float *st, const Chunk &c, float (&p)[kSteps])
{
    if (FROM_STATE) load_flat(st, c, g.n, p, 0.0f);
    else load_seg(g, c, p);
}

// ---------------------------------------------------------------------------
// plan (one block works) or refill (all blocks work), 1024 threads per block.
//
// plan: the candidates sit in per-chunk slots, very unevenly (a few tensors hold
// most of them).  One block scans the per-tile counts and lists the non-empty
// tiles with their running candidate numbers, cuts the candidate sequence into
// equal shares, one per wavefront of the later kernels, and resolves radix level 1.
//
// refill: runs instead if the hint left fewer than k candidates.  Every element
// becomes a candidate (chunk c holds candidates 1024 c ...), the elements below the
// hint join the level-1 histogram, and level 1 is resolved by the next kernel.
// ---------------------------------------------------------------------------
constexpr int kPlanThreads = 1024;
constexpr int kPlanPer = 16;          // tile counts a thread keeps in registers (covers 2^26 elements per group)

__device__ __forceinline__ uint32_t runs_total(uint64_t runs)
{
    return (uint32_t)(runs & 0xFFFFu) + (uint32_t)((runs >> 16) & 0xFFFFu) + (uint32_t)((runs >> 32) & 0xFFFFu) + (uint32_t)(runs >> 48);
}

template <bool FROM_STATE>
__global__ __launch_bounds__(kPlanThreads) void sparse_plan_k(GroupView g, const float *st, uint64_t k, uint32_t nwaves,
                                                              SparseScratch sc)
{
    __shared__ uint32_t hist[kBins1];
    __shared__ uint32_t wsum[kPlanThreads / 64];
    __shared__ uint32_t wsum_ne[kPlanThreads / 64];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t nch = (g.n + (uint32_t)kChunk - 1u) / (uint32_t)kChunk;
    const uint32_t ntiles = (g.n + (uint32_t)kTile - 1u) / (uint32_t)kTile;
    // ---- radix level 1 (need = k) from the bins the accumulate kernel filled: the last wavefront of block 0
    // does it while the others wait for their loads (after a refill the next kernel resolves again)
    if (blockIdx.x == 0 && wave == kPlanThreads / 64 - 1) {
        uint32_t bin;
        uint64_t rest;
        resolve_wave<kBins1>(sc.hist + kHist1, k, bin, rest);
        if (lane == 0) {
            SelectState s;
            s.prefix = bin << 20; s.pad0 = 0; s.need = rest;
            sc.sel[1] = s;
        }
    }
    // ---- every block: candidates and non-empty tiles before each thread's run of tiles
    const uint32_t per = (ntiles + kPlanThreads - 1) / kPlanThreads;
    const uint32_t lo = t * per < ntiles ? t * per : ntiles;
    const uint32_t hi = lo + per < ntiles ? lo + per : ntiles;
    const bool in_regs = per <= (uint32_t)kPlanPer;
    uint64_t r[kPlanPer];
    uint32_t own = 0, own_ne = 0;               // candidate numbers fit 32 bits: a group has fewer than 2^32 elements
    if (in_regs) {
#pragma unroll
        for (int i = 0; i < kPlanPer; ++i) r[i] = lo + i < hi ? sc.tile_runs[lo + i] : 0ull;   // all loads in flight at once
#pragma unroll
        for (int i = 0; i < kPlanPer; ++i) { own += runs_total(r[i]); own_ne += r[i] != 0ull; }
    } else {
        for (uint32_t c = lo; c < hi; ++c) { uint64_t x = sc.tile_runs[c]; own += runs_total(x); own_ne += x != 0ull; }
    }
    uint32_t incl = own, incl_ne = own_ne;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t a = __shfl_up(incl, d, 64), b = __shfl_up(incl_ne, d, 64);
        if (lane >= (uint32_t)d) { incl += a; incl_ne += b; }
    }
    if (lane == 63) { wsum[wave] = incl; wsum_ne[wave] = incl_ne; }
    __syncthreads();
    uint32_t p = incl - own, total = 0, q = incl_ne - own_ne, nonempty = 0;
#pragma unroll
    for (int w = 0; w < kPlanThreads / 64; ++w) {
        if ((uint32_t)w < wave) { p += wsum[w]; q += wsum_ne[w]; }
        total += wsum[w]; nonempty += wsum_ne[w];
    }
    if ((uint64_t)total >= k) {
        if (blockIdx.x != 0) return;
        // ---- plan
        const uint32_t share = total ? (total + nwaves - 1) / nwaves : 1u;
        auto place = [&](uint32_t tile, uint64_t runs) {
            if (runs) {
                const uint32_t cnt = runs_total(runs);
                sc.ne_tile[q] = tile;
                sc.ne_prefix[q] = p;
                sc.ne_runs[q] = runs;
                // wavefront j starts at candidate j * share: inside this tile if p <= j * share < p + cnt
                for (uint64_t j = (p + share - 1) / share; j * share < (uint64_t)p + cnt; ++j) sc.wave_start[j] = q;
                ++q;
                p += cnt;
            }
        };
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < kPlanPer; ++i) place(lo + i, r[i]);
        } else {
            for (uint32_t c = lo; c < hi; ++c) place(c, sc.tile_runs[c]);
        }
        if (t == 0) sc.ne_prefix[nonempty] = total;
        for (uint32_t j = t; j <= nwaves; j += kPlanThreads)
            if ((uint64_t)j * share >= total) sc.wave_start[j] = nonempty;
        if (t == 0) {
            PlanState pl;
            pl.total = total; pl.nonempty = nonempty; pl.share = share; pl.uniform = 0;
            *sc.plan = pl;
        }
        return;
    }
    // ---- refill
    for (int b = t; b < kBins1; b += kPlanThreads) hist[b] = 0u;
    __syncthreads();
    const uint32_t hint = *sc.hint;
    const uint32_t uwave = __builtin_amdgcn_readfirstlane(wave), waves = kPlanThreads / 64;
    for (uint32_t ch = blockIdx.x * waves + uwave; ch < nch; ch += gridDim.x * waves) {
        Chunk c;
        c.base = ch * (uint32_t)kChunk;
        c.lane = lane;
        c.full = g.n - c.base >= (uint32_t)kChunk;
        float v[kSteps];
        load_sel<FROM_STATE>(g, st, c, v);
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            uint32_t i = c.base + 64 * j + c.lane;
            if (c.full || i < g.n) {
                sc.cand_bits[i] = __float_as_uint(v[j]);
                sc.cand_loc[i] = (uint16_t)(64 * j + c.lane);
                if (key_of(v[j]) < hint) atomicAdd(&hist[key_of(v[j]) >> 20], 1u);
            }
        }
    }
    __syncthreads();
    flush_fine(hist, sc.hist + kHist1, kBins1);
    if (blockIdx.x == 0 && t == 0) {
        PlanState pl;
        pl.total = g.n; pl.nonempty = ntiles; pl.share = (g.n + nwaves - 1) / nwaves; pl.uniform = 1;
        *sc.plan = pl;
    }
}

// ---------------------------------------------------------------------------
// Walk one wavefront's share of the candidates, in index order.  The share is a
// range of candidate numbers; the plan says in which non-empty tile it starts.
// A window of 63 non-empty tiles (ids, first candidate numbers, per-chunk counts) is held
// in LDS; every lane finds its candidate's chunk by binary search there; four
// rounds of 64 candidates are fetched together, so the wavefront pays the memory
// latency once per 256 candidates.
// `body(valid, chunk, bits, loc)` is called by all 64 lanes (it may use ballots).
// ---------------------------------------------------------------------------
struct CandWindow { uint32_t first[64]; uint32_t tile[64]; uint64_t runs[64]; };

// A wavefront's share and the first window of its walk, fetched early so that the
// latency overlaps with whatever the kernel does before it walks.
struct CandCursor {
    uint64_t f_lo, f_hi;
    uint32_t uniform, nonempty, q0;
    uint32_t first, tile;      // this lane's entry of the first window
    uint64_t runs;
    bool active;
};

__device__ __forceinline__ void window_entry(const SparseScratch &sc, uint32_t n, const CandCursor &cur, uint32_t q0,
                                             uint32_t &first, uint32_t &tile, uint64_t &runs)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t q = q0 + lane < cur.nonempty ? q0 + lane : cur.nonempty;
    runs = 0;
    if (cur.uniform) { first = q < cur.nonempty ? q * (uint32_t)kTile : n; tile = q; }
    else {
        first = sc.ne_prefix[q];
        tile = q < cur.nonempty ? sc.ne_tile[q] : 0u;
        runs = q < cur.nonempty ? sc.ne_runs[q] : 0ull;
    }
}

__device__ __forceinline__ CandCursor cand_begin(const SparseScratch &sc, uint32_t n)
{
    CandCursor cur;
    const uint32_t w = blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t start = sc.wave_start[w];           // meaningless after a refill, then unused
    const uint64_t total = sc.plan->total;
    const uint32_t share = sc.plan->share;
    cur.uniform = sc.plan->uniform;
    cur.nonempty = sc.plan->nonempty;
    cur.f_lo = (uint64_t)w * share;
    cur.f_hi = cur.f_lo + share < total ? cur.f_lo + share : total;
    cur.active = cur.f_lo < total;
    cur.q0 = cur.uniform ? (uint32_t)(cur.f_lo >> 12) : start;
    cur.first = 0; cur.tile = 0; cur.runs = 0;
    if (cur.active) window_entry(sc, n, cur, cur.q0, cur.first, cur.tile, cur.runs);
    return cur;
}

template <bool WITH_LOC, typename Body>
__device__ __forceinline__ void cand_run(const CandCursor &cur, const SparseScratch &sc, uint32_t n,
                                         CandWindow *win /* LDS, per wavefront */, Body body)
{
    constexpr int kRounds = 4;
    if (!cur.active) return;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t uniform = cur.uniform;
    uint32_t q0 = cur.q0, first = cur.first, tile = cur.tile;
    uint64_t runs = cur.runs;
    for (;;) {
        __builtin_amdgcn_wave_barrier();
        win->first[lane] = first;
        win->tile[lane] = tile;
        win->runs[lane] = runs;
        __builtin_amdgcn_wave_barrier();
        const uint64_t win_lo = __builtin_amdgcn_readlane(first, 0), win_hi = __builtin_amdgcn_readlane(first, 63);
        const uint64_t a = cur.f_lo > win_lo ? cur.f_lo : win_lo, b = cur.f_hi < win_hi ? cur.f_hi : win_hi;
        for (uint64_t f0 = a; f0 < b; f0 += 64 * kRounds) {
            uint32_t ch[kRounds], bits[kRounds], loc[kRounds];
            size_t slot[kRounds];
            bool valid[kRounds];
#pragma unroll
            for (int u = 0; u < kRounds; ++u) {
                const uint64_t f = f0 + 64 * u + lane;
                valid[u] = f < b;
                const uint32_t f32 = (uint32_t)f;
                uint32_t ci = 0;
#pragma unroll
                for (int step = 32; step >= 1; step >>= 1)
                    if (valid[u] && win->first[ci + step] <= f32) ci += step;   // ci + step <= 63; f < first[63] keeps ci <= 62
                uint32_t off = valid[u] ? f32 - win->first[ci] : 0u;            // candidate number inside the tile
                uint32_t sub;                                                    // chunk of the tile, then slot inside it
                if (uniform) { sub = off >> 10; off &= 1023u; }
                else {
                    const uint64_t rr = win->runs[ci];
                    const uint32_t r0 = (uint32_t)(rr & 0xFFFFu), r1 = r0 + (uint32_t)((rr >> 16) & 0xFFFFu),
                                   r2 = r1 + (uint32_t)((rr >> 32) & 0xFFFFu);
                    sub = (off >= r0) + (off >= r1) + (off >= r2);
                    off -= sub == 0 ? 0u : sub == 1 ? r0 : sub == 2 ? r1 : r2;
                }
                ch[u] = win->tile[ci] * kWavesPerBlock + sub;
                slot[u] = valid[u] ? (size_t)ch[u] * kChunk + off : 0;
            }
#pragma unroll
            for (int u = 0; u < kRounds; ++u) {
                bits[u] = sc.cand_bits[slot[u]];
                loc[u] = WITH_LOC ? sc.cand_loc[slot[u]] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kRounds; ++u)
                if (f0 + 64 * u < b) body(valid[u], ch[u], bits[u], loc[u]);
        }
        if (win_hi >= cur.f_hi || q0 + 63 >= cur.nonempty) break;
        q0 += 63;
        window_entry(sc, n, cur, q0, first, tile, runs);
    }
}

// ---------------------------------------------------------------------------
// level 2 / level 3 histogram over the candidates
//   LEVEL 2: level 1 comes resolved from the plan (after a refill: resolved here, by the block),
//            histograms bits 19..10 of the matching keys
//   LEVEL 3: resolves level 2 (1024 bins, per wavefront), histograms bits 9..0
// Block 0 records the resolved prefix for the next kernel and clears the histogram
// that the previous kernel has finished reading.
// ---------------------------------------------------------------------------
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void cand_hist_k(uint32_t n, uint64_t k, SparseScratch sc)
{
    __shared__ uint32_t hist[1024];
    __shared__ CandWindow win[kWavesPerBlock];
    __shared__ uint64_t above[kBlock];
    __shared__ uint32_t res[3];
    for (int b = threadIdx.x; b < 1024; b += kBlock) hist[b] = 0u;
    const CandCursor cur = cand_begin(sc, n);
    uint32_t prefix;
    if (LEVEL == 2) {
        if (sc.plan->uniform) {                       // after a refill nobody has resolved level 1 yet
            resolve_block<kBins1, kBlock>(sc.hist + kHist1, k, above, res);
            prefix = res[0] << 20;
            if (blockIdx.x == 0 && threadIdx.x == 0) {
                SelectState s;
                s.prefix = prefix; s.pad0 = 0; s.need = (uint64_t)res[1] | ((uint64_t)res[2] << 32);
                sc.sel[1] = s;
            }
        } else prefix = sc.sel[1].prefix;
    } else {
        const SelectState s1 = sc.sel[1];
        uint32_t bin;
        uint64_t rest;
        resolve_wave<kBins2>(sc.hist + kHist2, s1.need, bin, rest);
        prefix = s1.prefix | (bin << 10);
        if (blockIdx.x == 0) {
            if (threadIdx.x == 0) {
                SelectState s;
                s.prefix = prefix; s.pad0 = 0; s.need = rest;
                sc.sel[2] = s;
            }
            for (int b = threadIdx.x; b < kHist2 - kHist1; b += kBlock) sc.hist[kHist1 + b] = 0u;   // level 2 is done with level 1
        }
    }
    __syncthreads();
    constexpr int kMatchShift = LEVEL == 2 ? 20 : 10;
    const uint32_t want = prefix >> kMatchShift;
    cand_run<false>(cur, sc, n, &win[threadIdx.x >> 6], [&](bool valid, uint32_t, uint32_t bits, uint32_t) {
        uint32_t key = bits & 0x7FFFFFFFu;
        if (valid && (key >> kMatchShift) == want) atomicAdd(&hist[(key >> (kMatchShift - 10)) & 1023u], 1u);
    });
    __syncthreads();
    flush_fine(hist, sc.hist + (LEVEL == 2 ? kHist2 : kHist3), 1024);
}

// ---------------------------------------------------------------------------
// count: resolve level 3 -> threshold key T and `need` (keys == T to take, in
// index order); kept candidates per wavefront and per block.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void cand_count_k(uint32_t n, SparseScratch sc)
{
    __shared__ uint32_t wgt[kWavesPerBlock], weq[kWavesPerBlock];
    __shared__ CandWindow win[kWavesPerBlock];
    const CandCursor cur = cand_begin(sc, n);
    const SelectState s2 = sc.sel[2];
    uint32_t bin;
    uint64_t rest;
    resolve_wave<kBins3>(sc.hist + kHist3, s2.need, bin, rest);
    const uint32_t T = s2.prefix | bin;
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            SelectState s;
            s.prefix = T; s.pad0 = 0; s.need = rest;
            sc.sel[3] = s;
            *sc.hint = T > kHintMargin ? T - kHintMargin : 0u;      // where the next call starts filtering
        }
        for (int b = threadIdx.x; b < kHist3 - kHist2; b += kBlock) sc.hist[kHist2 + b] = 0u;   // level 3 is done with level 2
    }
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t ngt = 0, neq = 0;
    cand_run<false>(cur, sc, n, &win[threadIdx.x >> 6], [&](bool valid, uint32_t, uint32_t bits, uint32_t) {
        uint32_t key = bits & 0x7FFFFFFFu;
        ngt += __popcll(__builtin_amdgcn_ballot_w64(valid && key > T));
        neq += __popcll(__builtin_amdgcn_ballot_w64(valid && key == T));
    });
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
__global__ __launch_bounds__(kBlock) void cand_emit_k(uint32_t n, float *st, PayloadHeader *hdr, uint64_t k, SparseScratch sc)
{
    __shared__ uint64_t sgt[kWavesPerBlock], seq[kWavesPerBlock];
    __shared__ CandWindow win[kWavesPerBlock];
    const SelectState s3 = sc.sel[3];
    const uint32_t T = s3.prefix;
    const uint64_t need = s3.need;
    uint32_t *idx = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(hdr) + kHeaderBytes);
    float *val = reinterpret_cast<float *>(idx + k);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    // kept-before of this block: sum over the blocks before it (at most 1024), four loads per thread
    uint32_t vg[4], ve[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint32_t b = u * kBlock + threadIdx.x;
        vg[u] = b < blockIdx.x ? sc.blk_gt[b] : 0u;
        ve[u] = b < blockIdx.x ? sc.blk_eq[b] : 0u;
    }
    const CandCursor cur = cand_begin(sc, n);       // its loads fly while the sums below are formed
    uint64_t ag = 0, ae = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) { ag += vg[u]; ae += ve[u]; }
    // kept-before of this wavefront inside the block
    uint64_t wg = 0, we = 0;
    if (lane < wave) {
        wg = sc.wave_gt[blockIdx.x * kWavesPerBlock + lane];
        we = sc.wave_eq[blockIdx.x * kWavesPerBlock + lane];
    }
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            PayloadHeader h;
            h.magic = kMagic; h.algo = ALGO; h.n = n; h.k = k; h.scale = 0.0f; h.levels = 0;
            for (int i = 0; i < 8; ++i) h.pad[i] = 0;
            *hdr = h;
        }
        for (int b = threadIdx.x; b < kHistWords - kHist3; b += kBlock) sc.hist[kHist3 + b] = 0u;   // count is done with level 3
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        ag += __shfl_xor(ag, m, 64); ae += __shfl_xor(ae, m, 64);
        wg += __shfl_xor(wg, m, 64); we += __shfl_xor(we, m, 64);
    }
    if (lane == 0) { sgt[wave] = ag; seq[wave] = ae; }
    __syncthreads();
    uint64_t gt_before = (sgt[0] + sgt[1]) + (sgt[2] + sgt[3]) + wg;
    uint64_t eq_before = (seq[0] + seq[1]) + (seq[2] + seq[3]) + we;
    cand_run<true>(cur, sc, n, &win[wave], [&](bool valid, uint32_t chunk, uint32_t b, uint32_t loc) {
        const uint32_t key = b & 0x7FFFFFFFu;
        const bool is_gt = valid && key > T, is_eq = valid && key == T;
        const uint64_t bgt = __builtin_amdgcn_ballot_w64(is_gt), beq = __builtin_amdgcn_ballot_w64(is_eq);
        const uint64_t gtb = gt_before + lanes_below(bgt), eqb = eq_before + lanes_below(beq);
        if (is_gt || (is_eq && eqb < need)) {
            const uint64_t pos = gtb + (eqb < need ? eqb : need);
            const uint32_t i = chunk * (uint32_t)kChunk + loc;
            if (pos < k && i < n) {                  // always true for consistent scratch; guards the buffers
                idx[pos] = i;
                val[pos] = __uint_as_float(b);
                if (ALGO == MC_ALGO_DGC) { st[i] = 0.0f; st[(size_t)n + i] = 0.0f; }   // momentum factor masking
                else if (EF) st[i] = 0.0f;
            }
        }
        gt_before += __popcll(bgt);
        eq_before += __popcll(beq);
    });
}

// grid of the kernels that walk the candidates: one wavefront per share, at most kMaxCandBlocks blocks
static inline uint32_t cand_blocks(uint32_t nchunks)
{
    uint32_t b = (nchunks + kWavesPerBlock - 1) / kWavesPerBlock;
    if (b < 1) b = 1;
    return b < kMaxCandBlocks ? b : kMaxCandBlocks;
}

template <int ALGO, bool EF>
static void sparse_compress_t(const LaunchCtx &lc, const GroupView &g, float *st, float momentum, uint64_t k,
                              PayloadHeader *hdr, const SparseScratch &sc)
{
    constexpr bool FS = (ALGO == MC_ALGO_DGC) || EF;
    const uint32_t nt = tiles_of(g.n), nch = chunks_of(g.n);
    const uint32_t cblocks = cand_blocks(nch), nwaves = cblocks * kWavesPerBlock;
    const uint32_t pblocks = (nch + 15) / 16 < 256 ? (nch + 15) / 16 : 256;
    dim3 grid(nt), block(kBlock), cgrid(cblocks);
    prof_begin(lc, K_SPARSE_ACCUM);
    MC_LAUNCH((sparse_accum_k<ALGO, EF>), grid, block, lc, g, st, momentum, sc);
    prof_end(lc, K_SPARSE_ACCUM);
    prof_begin(lc, K_SPARSE_PLAN);
    MC_LAUNCH(sparse_plan_k<FS>, dim3(pblocks), dim3(kPlanThreads), lc, g, st, k, nwaves, sc);
    prof_end(lc, K_SPARSE_PLAN);
    prof_begin(lc, K_CAND_HIST);
    MC_LAUNCH(cand_hist_k<2>, cgrid, block, lc, g.n, k, sc);
    prof_end(lc, K_CAND_HIST);
    prof_begin(lc, K_CAND_HIST);
    MC_LAUNCH(cand_hist_k<3>, cgrid, block, lc, g.n, k, sc);
    prof_end(lc, K_CAND_HIST);
    prof_begin(lc, K_CAND_COUNT);
    MC_LAUNCH(cand_count_k, cgrid, block, lc, g.n, sc);
    prof_end(lc, K_CAND_COUNT);
    prof_begin(lc, K_CAND_EMIT);
    MC_LAUNCH((cand_emit_k<ALGO, EF>), cgrid, block, lc, g.n, st, hdr, k, sc);
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
// output tile owns one contiguous run of each list.  A first kernel records, per
// worker and tile, where that run starts and ends (one thread per payload entry, no
// search; entries are stamped with a per-call epoch instead of clearing the table);
// the second accumulates each tile in LDS, one worker after the other in ascending
// worker order -- the same order of fp32 additions as a dense sum, since adding
// the +0 of an absent entry changes nothing -- and writes it once.  No atomics, no
// pre-zeroed output, bit-reproducible.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void sparse_index_k(int algo, uint32_t n, PayloadPtrs pl, int W, uint64_t k64,
                                                         uint32_t ntiles, uint32_t epoch, uint64_t *tile_first,
                                                         uint64_t *tile_last, int *status)
{
    const uint32_t k = (uint32_t)k64;
    const uint32_t w = blockIdx.y;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const PayloadHeader *h = reinterpret_cast<const PayloadHeader *>(pl.p[w]);
        if (h->magic != kMagic || h->algo != (uint32_t)algo || h->n != (uint64_t)n || h->k != k64) *status = 1;
    }
    const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w] + kHeaderBytes);
    const uint32_t e = blockIdx.x * kBlock + threadIdx.x;
    if (e >= k) return;
    // the first entry of a tile's run records where the run starts, the last one where it ends;
    // both are stamped with this call's epoch, so tiles without entries need no clearing
    const uint32_t tile = idx[e] >> 12;
    if (tile >= ntiles) return;
    const uint64_t stamp = (uint64_t)epoch << 32;
    if (e == 0 || (idx[e - 1] >> 12) != tile) tile_first[(size_t)w * ntiles + tile] = stamp | e;
    if (e == k - 1 || (idx[e + 1] >> 12) != tile) tile_last[(size_t)w * ntiles + tile] = stamp | (e + 1);
}

constexpr int kSparseBatch = 8;    // workers whose entries are in flight together
constexpr int kSparseRounds = 4;   // rounds of 256 entries per worker fetched up front

__global__ __launch_bounds__(kBlock) void sparse_decompress_k(GroupView out, PayloadPtrs pl, int W, float alpha,
                                                              uint64_t k64, uint32_t ntiles, uint32_t epoch,
                                                              const uint64_t *tile_first, const uint64_t *tile_last)
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
                const uint64_t f = tile_first[(size_t)(w0 + b) * ntiles + blockIdx.x];
                const uint64_t l = tile_last[(size_t)(w0 + b) * ntiles + blockIdx.x];
                if ((uint32_t)(f >> 32) == epoch && (uint32_t)(l >> 32) == epoch) {      // else: no entry in this tile
                    lo[b] = (uint32_t)f < k ? (uint32_t)f : k;
                    hi[b] = (uint32_t)l < k ? (uint32_t)l : k;
                    // inconsistent payload (indices not ascending): a tile holds at most 4096 entries
                    if (hi[b] < lo[b] || hi[b] - lo[b] > (uint32_t)kTile) hi[b] = lo[b];
                }
            }
        }
        if (W <= kSparseBatch) {          // most tiles hold no kept entry at all: they are just zero-filled
            bool any = false;
#pragma unroll
            for (int b = 0; b < kSparseBatch; ++b) any = any || hi[b] > lo[b];
            if (!any) {
                const Chunk c = my_chunk(out.n);
                if (c.base >= out.n) return;
                float z[kSteps];
#pragma unroll
                for (int j = 0; j < kSteps; ++j) z[j] = alpha * 0.0f;
                store_seg(out, c, z);
                return;
            }
        }
        // the kept entries cluster in a few tensors: a tile there holds hundreds of entries per worker.
        // Four rounds of 256 entries of every worker of the batch are requested at once.
        uint32_t ix[kSparseBatch][kSparseRounds];
        float vv[kSparseBatch][kSparseRounds];
#pragma unroll
        for (int b = 0; b < kSparseBatch; ++b) {
            const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w0 + b < W ? w0 + b : 0] + kHeaderBytes);
            const float *val = reinterpret_cast<const float *>(idx + k);
#pragma unroll
            for (int r = 0; r < kSparseRounds; ++r) {
                const uint32_t e = lo[b] + r * kBlock + t;
                ix[b][r] = 0xFFFFFFFFu; vv[b][r] = 0.0f;
                if (w0 + b < W && e < hi[b]) { ix[b][r] = ld_stream(idx + e); vv[b][r] = ld_stream(val + e); }
            }
        }
#pragma unroll
        for (int b = 0; b < kSparseBatch; ++b) {
            if (w0 + b < W) {
#pragma unroll
                for (int r = 0; r < kSparseRounds; ++r) {
                    const uint32_t local = ix[b][r] - tb;
                    if (ix[b][r] != 0xFFFFFFFFu && local < (uint32_t)kTile) acc[local] = acc[local] + vv[b][r];
                }
                // more than 1024 entries of one worker in the tile
                const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[w0 + b] + kHeaderBytes);
                const float *val = reinterpret_cast<const float *>(idx + k);
                for (uint32_t e = lo[b] + kSparseRounds * kBlock + t; e < hi[b]; e += kBlock) {
                    const uint32_t l2 = idx[e] - tb;
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
                              float alpha, uint64_t k, uint32_t epoch, uint64_t *tile_first, uint64_t *tile_last, int *status)
{
    if (out.n == 0) return;
    const uint32_t nt = tiles_of(out.n);
    prof_begin(lc, K_SPARSE_INDEX);
    MC_LAUNCH(sparse_index_k, dim3((uint32_t)((k + kBlock - 1) / kBlock), W), dim3(kBlock), lc, algo,
                       out.n, pl, W, k, nt, epoch, tile_first, tile_last, status);
    prof_end(lc, K_SPARSE_INDEX);
    prof_begin(lc, K_SPARSE_DECOMPRESS);
    MC_LAUNCH(sparse_decompress_k, dim3(nt), dim3(kBlock), lc, out, pl, W, alpha, k, nt, epoch, tile_first,
                       tile_last);
    prof_end(lc, K_SPARSE_DECOMPRESS);
}

}  // namespace mc
