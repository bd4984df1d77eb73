// Sparsifiers (Top-k, DGC, Rand-k) for gfx950: exact top-k of |p| over a whole merged
// group, ties at the threshold taken in index order (lower index wins), payload
// written in ascending index order, and the sparse decompress-and-sum.
// Rand-k is the same selection on keys that do not depend on the values: the k
// largest of the elements' Philox words (31 bits) are k positions drawn uniformly.
//
// The paper singles out the top-k() operation as the cost that merging alone
// does not remove (Section 5.1).  Here the selection is a radix select on the
// 31-bit magnitude key that never sorts and, in the steady state, touches the
// gradient once and resolves 20 of the 31 bits inside that one pass:
//
//   accumulate   p = g + e (DGC: u = m u + g, v = v + u) streamed once; every element
//                whose key reaches a *hint* (a little below the last threshold of this
//                group) is copied, in index order, into the candidate slots of its
//                1024-element chunk, and counted in a *window* histogram: 2048 bins of
//                2048 keys each, starting at the hint (the last bin also takes all above)
//   seed         reads the window.  Usual case: the k-th largest key falls in one of its
//                bins, which leaves 11 bits to resolve (fast mode).  Otherwise all blocks
//                build a level-1 histogram (top 11 bits of key - lo) of the candidates
//                above the window, or, if the hint left fewer than k candidates (first
//                call, or the distribution moved down), of every element (refill)
//   hist 2       only after a seed that was not fast: bits 19..10 of key - lo
//   hist 3       the bits still open (11 after a fast seed, else 10)
//   count        resolves level 3 (threshold key T, number of keys == T to take),
//                counts kept candidates per tile, publishes the next hint
//   emit         ordered compaction of the kept candidates into (idx, val); kept
//                entries leave the residual
//
// If at least k elements have key >= hint, the k-th largest key T is >= hint, so
// every element with key >= T is a candidate and the result is exact whatever the
// hint was; the hint only decides how much work the later kernels have.
// The kernels that walk the candidates give every 4096-element tile to one
// wavefront: tiles are independent until the emit kernel adds up the kept counts
// of the tiles before its own.  No kernel waits on another block: every dependency
// is a kernel boundary.
#include <algorithm>

#include "mc_internal.h"

namespace mc {

static inline uint32_t tiles_of(uint32_t n) { return (uint32_t)(((uint64_t)n + kTile - 1) / kTile); }
static inline uint32_t chunks_of(uint32_t n) { return (uint32_t)(((uint64_t)n + kChunk - 1) / kChunk); }

constexpr int kWindowShift = 11;                       // keys per window bin = 2^11: what hist 3 resolves after a fast seed
constexpr int kBinsW = 2048, kBins1 = 2048, kBins2 = 1024, kBins3 = 1 << kWindowShift;
// Histogram scratch: the window and the three radix levels one after the other.  Global
// atomics on one address serialise (tens of nanoseconds each on this part), so only
// the bins themselves are updated -- no shared summary counters -- and a level is
// resolved by a wavefront that reads all its bins.
// The window histogram is kept in kWinCopies copies, a block adding to the copy of its index, and the seed sums
// them.  The flush of the streaming pass is one multi-lane add per block and 128-byte line of bins, and adds to one
// line queue up behind each other (about 5 ns each): when the candidates are spread evenly over the tiles, every
// block holds some of nearly every bin between the hint and the threshold, and with a single copy the pass took
// 132 us instead of 54 (all tensors of one scale).  One bin per line was tried first (62 us, but the adds of a wave
// no longer coalesce: +2..4 us on clustered candidates and a 2048-line gather in the seed); copies keep the adds
// coalesced.  Measured, Top-k compress on clustered / evenly spread candidates: 2 copies 87.6 / 125.6 us, 4 copies
// 88.4 / 97.5, 8 copies 89.7 / 99.0, 16 copies 93.3 / 101.7, 32 copies 106 / 114 (the seed reads them all).
constexpr int kHistW = 0, kHist1 = kHistW + kBinsW * kWinCopies, kHist2 = kHist1 + kBins1, kHist3 = kHist2 + kBins2;
// The window's open last bin takes a count from nearly every block (all keys above the window), and
// adds from thousands of blocks to one address queue up behind each other for tens of microseconds:
// its count is spread over kOpenCopies words, chosen by the block index, which the seed sums.
constexpr int kOpenCopies = 64, kHistOpen = kHist3 + kBins3;
static_assert(kHistOpen + kOpenCopies == kHistWords, "histogram scratch layout");
constexpr uint32_t kHintMargin = 3u << 19;   // 3/16 of an octave below the last threshold
// The window spans 2^22 keys (half an octave) from the hint upward: it holds the new threshold if that
// lies between 12 % below and 24 % above the last one (2^23 keys are one octave of magnitude).

// seed result (SelectState::mode)
// hint record of a (group, worker): the filter key, how many times the margin below the threshold was halved,
// and for how many calls it stays at the full margin after a miss
constexpr int kHintShift = 1, kHintHold = 2, kHintCap = 3;
constexpr uint32_t kHintShiftMax = 4u, kHintHoldCalls = 8u;      // margin at least 3/256 of an octave (0.8 %)
constexpr uint32_t kHintCapCalls = 64u;

// How far below the threshold the next call starts filtering, after a call whose threshold lay inside the window.
// Under error feedback the values pile up just below the threshold, in the long run those of every tensor, and a fixed
// margin lets through many times k of them (each costs the streaming pass a store and the histogram an add): the
// margin is halved while the filter passes more than 2 k (at most four times: 0.8 % below the threshold) and doubled
// again when it passes fewer than 1.25 k.  (Measured, every worker on new gradients: with "more than 4 k" the bench's
// Top-k stayed at the full margin, 12 %, and 850 000 candidates; with 3 k it settles at one halving and 533 000,
// with 2 k at two, 3 %, and 396 000: Top-k compress went 80.2 -> 78.5 us with the second rule and 77.0 -> 75.5 us
// with the third, no miss in 200 calls with any of them.)
// A call whose threshold fell below the filter (a miss: a second streaming pass) resets the margin, keeps it for
// kHintHoldCalls calls, and caps the halvings below what the margin had been halved to when it missed, one step
// more being allowed again after every kHintCapCalls calls: a threshold that jitters by more than the tightest margin
// costs a miss every so many calls, not every few.  cap word: steps taken off kHintShiftMax | calls left << 8.
__device__ __forceinline__ void margin_after_hit(uint32_t *hint, uint32_t shift, uint32_t hold, uint32_t capw, uint64_t cands, uint64_t k)
{
    uint32_t off = capw & 0xFFu, left = capw >> 8;
    if (left) --left;
    else if (off) { --off; left = off ? kHintCapCalls : 0u; }
    const uint32_t cap = kHintShiftMax - (off < kHintShiftMax ? off : kHintShiftMax);
    if (hold) --hold;
    else if (cands > 2u * k && shift < cap) ++shift;
    if (4u * cands < 5u * k && shift) --shift;
    if (shift > cap) shift = cap;
    hint[kHintShift] = shift; hint[kHintHold] = hold; hint[kHintCap] = off | (left << 8);
}
// below: the threshold fell below the filter (else it rose above the window, which no margin prevents)
__device__ __forceinline__ void margin_after_miss(uint32_t *hint, uint32_t shift, bool below)
{
    hint[kHintShift] = 0u; hint[kHintHold] = kHintHoldCalls;
    if (below && shift) hint[kHintCap] = (kHintShiftMax - (shift - 1u)) | (kHintCapCalls << 8);
}
constexpr uint32_t kModeFast = 1u;      // lo / need are those of level 3 already
constexpr uint32_t kModeUniform = 2u;   // after a refill: every element is a candidate, chunk c holds 1024 c ...
constexpr uint32_t kModeLean = 4u;      // fast, and the keys of the threshold's window bin were listed: the emit kernel finishes alone
constexpr uint32_t kModeDense = 8u;     // fast, but that bin holds too many keys to list: its 2048 keys were histogrammed instead

__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// add a block's LDS histogram to the global one
__device__ __forceinline__ void flush_fine(const uint32_t *lds, uint32_t *fine, int bins)
{
    for (int b = threadIdx.x; b < bins; b += blockDim.x) {
        uint32_t h = lds[b];
        if (h) atomicAdd(&fine[b], h);
    }
}

// key of the stochastic choices: Philox key and the worker / iteration words of the counter
struct RngKey { uint64_t seed; uint32_t worker, iter_lo; };

// DGC with a sampled threshold: the histograms that find the threshold count only the sample, every
// stride-th element of the group starting at `first` (drawn by the host with Philox).  stride = 0: off.
struct SampleRule { uint32_t stride, first, inv /* floor(2^32 / stride) */; };

__device__ __forceinline__ bool in_sample(const SampleRule &r, uint32_t i)
{
    if (r.stride <= 1u) return true;
    uint32_t rem = i - __umulhi(i, r.inv) * r.stride;      // the quotient estimate is at most 1 too small
    if (rem >= r.stride) rem -= r.stride;
    return rem == r.first;
}

// Copy the flagged elements of a chunk, in index order, into the chunk's candidate slots.
// bits: what the later kernels see of the element (its key is bits & 0x7FFFFFFF): the value itself, or
// for Rand-k the random key.
__device__ __forceinline__ uint32_t put_candidates(const Chunk &c, const uint32_t (&bits)[kSteps], const uint64_t (&flag)[kSteps],
                                                   uint32_t hint, uint32_t *cand_bits, uint16_t *cand_loc, uint32_t *hist /* LDS */,
                                                   const SampleRule &smp)
{
    uint32_t run = 0;
    const uint64_t me = 1ull << c.lane;
#pragma unroll
    for (int j = 0; j < kSteps; ++j) {
        if (flag[j] & me) {
            uint32_t slot = c.base + run + lanes_below(flag[j]);
            cand_bits[slot] = bits[j];
            cand_loc[slot] = (uint16_t)(64 * j + c.lane);
            const uint32_t bin = ((bits[j] & 0x7FFFFFFFu) - hint) >> kWindowShift;
            if (in_sample(smp, c.base + 64 * j + c.lane))
                atomicAdd(&hist[bin < (uint32_t)kBinsW - 1u ? bin : (uint32_t)kBinsW - 1u], 1u);
        }
        run += __popcll(flag[j]);
    }
    return run;
}

// ---------------------------------------------------------------------------
// accumulate + candidate filter + window histogram of the candidates
// ---------------------------------------------------------------------------
template <int ALGO, bool EF>
__global__ __launch_bounds__(kBlock) void sparse_accum_k(GroupView g, float *st, float momentum, SparseScratch sc, RngKey rng,
                                                         SampleRule smp)
{
    __shared__ uint32_t hist[kBinsW];
    __shared__ uint32_t wcnt[kWavesPerBlock];
    for (int b = threadIdx.x; b < kBinsW; b += kBlock) hist[b] = 0u;
    __syncthreads();
    const Chunk c = my_chunk(g.n);
    const uint32_t hint = *sc.hint;
    // the emit kernel of the call before is done with the list of keys in the threshold's bin: its sublists are empty again
    if (blockIdx.x == 0 && threadIdx.x < (uint32_t)kUSub) sc.ucount[threadIdx.x * kUCountStride] = 0u;
    if (blockIdx.x == 0 && threadIdx.x == 0) sc.sync[0] = 0u;       // and nobody waits at a grid-wide barrier of that call any more
    // The radix levels are cleared by the kernels that use them -- unless a call gave up at a barrier (MC_ERR_DEVICE):
    // what it left behind must not enter this call's counts.
    {
        const uint32_t i = blockIdx.x * (uint32_t)kBlock + threadIdx.x;
        if (i < (uint32_t)(kHistOpen - kHist1)) sc.hist[kHist1 + i] = 0u;
    }
    uint32_t run = 0;
    if (c.base < g.n) {
        float p[kSteps];
        // What the last call sent leaves the memory: an element whose key was above that call's threshold key counts as 0
        // here, instead of having been set to 0 there -- one scattered 4-byte store per kept entry, each a read-modify-write
        // of a whole line in memory, was most of what the compaction cost.  (Kept entries *equal* to the threshold are still
        // zeroed in place: which of the equal keys were taken depends on their order.  A state that was zero-filled,
        // imported, or written by a scheme that zeroes in place says sent_key = all ones or holds zeros: nothing is masked.)
        const uint32_t sent_key = (ALGO == MC_ALGO_DGC || EF) ? reinterpret_cast<const StateHeader *>(reinterpret_cast<const uint8_t *>(st) - kHeaderBytes)->sent_key : 0u;
        if (ALGO == MC_ALGO_DGC) {
            // momentum correction: u = m u + g ; v = v + u ; the vector compressed is v
            float *vbuf = st, *ubuf = st + dgc_u_offset(g.n);
            float u[kSteps], v[kSteps];
            load_flat(ubuf, c, g.n, u, 0.0f);
            load_flat(vbuf, c, g.n, v, 0.0f);
            load_seg(g, c, p);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                if (key_of(v[j]) > sent_key) { u[j] = 0.0f; v[j] = 0.0f; }       // momentum factor masking of what was sent
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
            for (int j = 0; j < kSteps; ++j) p[j] = p[j] + (key_of(e[j]) > sent_key ? 0.0f : e[j]);
            store_flat(st, c, g.n, p);
        } else {
            load_seg(g, c, p);
        }
        uint32_t bits[kSteps];
        if (ALGO == MC_ALGO_RANDK) {
            chunk_words(rng.seed, rng.worker, rng.iter_lo, g.goff + c.base, c.lane, bits);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) bits[j] >>= 1;
        } else {
#pragma unroll
            for (int j = 0; j < kSteps; ++j) bits[j] = __float_as_uint(p[j]);
        }
        uint64_t flag[kSteps];
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            bool valid = c.full || c.base + 64 * j + c.lane < g.n;
            flag[j] = __builtin_amdgcn_ballot_w64(valid && (bits[j] & 0x7FFFFFFFu) >= hint);
        }
        run = put_candidates(c, bits, flag, hint, sc.cand_bits, sc.cand_loc, hist, smp);
    }
    if (c.lane == 0) wcnt[threadIdx.x >> 6] = run;
    __syncthreads();
    if (threadIdx.x == 0)       // candidates of the tile's four chunks, 16 bits each (a chunk holds at most 1024)
        sc.tile_runs[my_tile_index()] = (uint64_t)wcnt[0] | ((uint64_t)wcnt[1] << 16) | ((uint64_t)wcnt[2] << 32) | ((uint64_t)wcnt[3] << 48);
    flush_fine(hist, sc.hist + kHistW + (blockIdx.x % kWinCopies) * kBinsW, kBinsW - 1);
    if (threadIdx.x == kBlock - 1 && hist[kBinsW - 1]) atomicAdd(&sc.hist[kHistOpen + (blockIdx.x & (kOpenCopies - 1))], hist[kBinsW - 1]);
}

// ---------------------------------------------------------------------------
// Resolve one radix level inside a wavefront: find the bin b with
//   count(bins > b) < need <= count(bins >= b)        and  rest = need - count(bins > b).
// Every lane reads BINS / 64 adjacent bins, a suffix scan over the lanes finds the
// lane where the running count crosses `need`, and that lane walks its own bins.
// One memory latency, no block barrier.  Returns false (bin = 0, rest = 0) if the
// histogram holds fewer than `need` keys.
// ---------------------------------------------------------------------------
template <int BINS>
__device__ __forceinline__ bool resolve_wave(const uint32_t *fine, uint64_t need, uint32_t &bin, uint64_t &rest,
                                             uint32_t top_extra = 0u /* counted in the last bin besides fine[BINS - 1] */,
                                             uint64_t *total = nullptr /* out: the sum of all bins */)
{
    constexpr int kPer = BINS / 64;
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t h[kPer];
    uint64_t own = 0;
    const uint4 *src = reinterpret_cast<const uint4 *>(fine + lane * kPer);
#pragma unroll
    for (int i = 0; i < kPer / 4; ++i) {
        const uint4 x = src[i];
        h[4 * i] = x.x; h[4 * i + 1] = x.y; h[4 * i + 2] = x.z; h[4 * i + 3] = x.w;
    }
    if (lane == 63u) h[kPer - 1] += top_extra;
#pragma unroll
    for (int i = 0; i < kPer; ++i) own += h[i];
    uint64_t incl = own;                                    // inclusive suffix sum over lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t o = __shfl_down(incl, d, 64);
        if (lane + d < 64) incl += o;
    }
    if (total) *total = __shfl(incl, 0, 64);
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
    const uint32_t src_lane = hit ? (uint32_t)__builtin_ctzll(hit) : 0u;     // an inconsistent histogram still gives a defined bin
    bin = __shfl(b, src_lane, 64);
    rest = __shfl(r, src_lane, 64);
    return hit != 0;
}

// The same for a histogram in LDS.  There the adjacent bins of a lane would all fall into the banks that every
// other lane's bins fall into (a lane owns BINS / 64 = 32 consecutive words: 64 lanes, one bank group), and the
// reads of a wavefront would be served one lane at a time -- measured: the resolve of a 2048-bin histogram by
// all four wavefronts of all blocks made the emit kernel twice as long.  Each lane therefore reads its bins in
// an order rotated by its lane number, which spreads every read over all banks; the lane in which the count
// crosses `need` reads its bins once more, in order.
template <int BINS>
__device__ __forceinline__ bool resolve_lds(const uint32_t *fine, uint64_t need, uint32_t &bin, uint64_t &rest,
                                            uint32_t top_extra = 0u, uint64_t *total = nullptr)
{
    constexpr int kPer = BINS / 64;
    static_assert((kPer & (kPer - 1)) == 0, "rotation needs a power of two");
    const uint32_t lane = threadIdx.x & 63u;
    uint64_t own = 0;
#pragma unroll 4              // (a few reads in flight are enough; all 32 at once cost the calling kernel its registers)
    for (int i = 0; i < kPer; ++i) own += fine[lane * kPer + ((i + lane) & (kPer - 1))];
    if (lane == 63u) own += top_extra;
    uint64_t incl = own;                                    // inclusive suffix sum over lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t o = __shfl_down(incl, d, 64);
        if (lane + d < 64) incl += o;
    }
    if (total) *total = __shfl(incl, 0, 64);
    uint64_t run = incl - own;                              // keys in the bins of higher lanes
    const bool mine = run < need && need <= incl;
    uint32_t b = 0;
    uint64_t r = 0;
    if (mine) {
        for (int i = kPer - 1; i >= 0; --i) {
            const uint64_t h = (uint64_t)fine[lane * kPer + i] + (lane == 63u && i == kPer - 1 ? top_extra : 0u);
            if (run < need && need <= run + h) { b = lane * kPer + i; r = need - run; }
            run += h;
        }
    }
    const uint64_t hit = __builtin_amdgcn_ballot_w64(mine);
    const uint32_t src_lane = hit ? (uint32_t)__builtin_ctzll(hit) : 0u;
    bin = __shfl(b, src_lane, 64);
    rest = __shfl(r, src_lane, 64);
    return hit != 0;
}

// the vector the selection works on: v / p kept in the state, or the gradient itself
template <bool FROM_STATE>
__device__ __forceinline__ void load_sel(const GroupView &g, const float *st, const Chunk &c, float (&p)[kSteps])
{
    if (FROM_STATE) load_flat(st, c, g.n, p, 0.0f);
    else load_seg(g, c, p);
}

// ---------------------------------------------------------------------------
// The candidates of one tile, walked by one wavefront in index order.  `runs`
// holds the candidate counts of the tile's four chunks (16 bits each); the slots of
// chunk c are cand[1024 c ...].  Up to twelve rounds of 64 candidates are fetched together,
// so a tile of a tensor that holds most of the kept entries (several hundred
// candidates) costs the wavefront one memory latency.
// `body(valid, chunk, bits, loc)` is called by all 64 lanes (it may use ballots).
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t runs_total(uint64_t runs)
{
    return (uint32_t)(runs & 0xFFFFu) + (uint32_t)((runs >> 16) & 0xFFFFu) + (uint32_t)((runs >> 32) & 0xFFFFu) + (uint32_t)(runs >> 48);
}

// candidate counts of a tile after a refill: every element below n
__device__ __forceinline__ uint64_t uniform_runs(uint32_t tile, uint32_t n)
{
    uint64_t r = 0;
#pragma unroll
    for (int s = 0; s < kWavesPerBlock; ++s) {
        const uint64_t base = (uint64_t)tile * kTile + (uint64_t)s * kChunk;
        const uint64_t cnt = base >= n ? 0u : (n - base < (uint64_t)kChunk ? n - base : (uint64_t)kChunk);
        r |= cnt << (16 * s);
    }
    return r;
}

// One batch of the walk: rounds [f0, f0 + 64 ROUNDS) of the tile's candidates, all loads issued before the first use.
template <bool WITH_LOC, int ROUNDS, typename Body>
__device__ __forceinline__ void tile_batch(const SparseScratch &sc, uint32_t tile, uint32_t r0, uint32_t r1, uint32_t r2, uint32_t total,
                                           uint32_t f0, Body body)
{
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t ch[ROUNDS], bits[ROUNDS], loc[ROUNDS];
    size_t slot[ROUNDS];
    bool valid[ROUNDS];
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        const uint32_t f = f0 + 64 * u + lane;
        valid[u] = f < total;
        const uint32_t sub = (f >= r0) + (f >= r1) + (f >= r2);          // chunk of the tile, then slot inside it
        const uint32_t off = f - (sub == 0 ? 0u : sub == 1 ? r0 : sub == 2 ? r1 : r2);
        ch[u] = tile * kWavesPerBlock + (valid[u] ? sub : 0u);
        slot[u] = valid[u] ? (size_t)ch[u] * kChunk + off : (size_t)tile * kTile;
    }
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        bits[u] = 0u; loc[u] = 0u;
        if (valid[u]) {
            bits[u] = sc.cand_bits[slot[u]];
            if (WITH_LOC) loc[u] = sc.cand_loc[slot[u]];
        }
    }
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u)
        if (f0 + 64 * u < total) body(valid[u], ch[u], bits[u], loc[u]);
}

// A tile with at most 256 candidates -- nearly every tile when the candidates are spread over the whole group -- takes
// one batch of four rounds: the slot arithmetic of sixteen rounds, most of them empty, was a third of what the
// count kernel did.  Other tiles take batches of twelve rounds (with sixteen the level-3 and emit kernels need 81 .. 83
// registers and five wavefronts fit a SIMD; with twelve, seven or eight do; eight rounds measure the same but would
// cost a tile full of candidates eight dependent batches).  Top-k compress, evenly spread / clustered candidates:
// 98.2 -> 89.7 us / 88.6 -> 88.1; Rand-k 97.7 -> 90.0; DGC 114.1 -> 111.4.
// Fetching the four rounds ahead of what else a kernel waits for (its resolve, its prefix sum) gained another 1 us on
// spread candidates and lost as much on clustered ones, whose heavy tiles then wait for their candidate counts before
// anything else is asked for: not kept.
template <bool WITH_LOC, typename Body>
__device__ __forceinline__ void tile_walk(const SparseScratch &sc, uint32_t tile, uint64_t runs, Body body)
{
    constexpr int kRounds = 12, kFew = 4;
    const uint32_t r0 = (uint32_t)(runs & 0xFFFFu), r1 = r0 + (uint32_t)((runs >> 16) & 0xFFFFu),
                   r2 = r1 + (uint32_t)((runs >> 32) & 0xFFFFu), total = r2 + (uint32_t)(runs >> 48);
    if (total <= 64u * kFew) { tile_batch<WITH_LOC, kFew>(sc, tile, r0, r1, r2, total, 0u, body); return; }
    for (uint32_t f0 = 0; f0 < total; f0 += 64 * kRounds) tile_batch<WITH_LOC, kRounds>(sc, tile, r0, r1, r2, total, f0, body);
}

// the tile of this wavefront in the kernels that walk the candidates, and its runs
struct TileJob { uint32_t tile; uint64_t runs; };

__device__ __forceinline__ TileJob my_tile(const SparseScratch &sc, uint32_t n, uint32_t ntiles)
{
    TileJob j;
    j.tile = blockIdx.x * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    j.runs = j.tile < ntiles ? sc.tile_runs[j.tile] : 0ull;      // ignored after a refill
    return j;
}

// ---------------------------------------------------------------------------
// seed: 1024 threads per block.  Wavefront 0 of every block resolves the window
// histogram; all blocks reach the same verdict.
//   fast      the threshold lies in window bin b < 2047: block 0 records lo = hint + 2048 b
//             and the entries to take from that bin; everybody leaves
//   above     it lies above the window: all blocks histogram bits 30..20 of key - lo of
//             the candidates with key >= lo = hint + 2048 * 2047
//   refill    fewer than k candidates: every element becomes a candidate (chunk c holds
//             candidates 1024 c ...) and joins the level-1 histogram of the plain keys
// ---------------------------------------------------------------------------
constexpr int kSeedThreads = 1024;

template <bool FROM_STATE, bool RANDOM>
__global__ __launch_bounds__(kSeedThreads) void sparse_seed_k(GroupView g, const float *st, uint64_t k, SparseScratch sc, RngKey rng,
                                                              SampleRule smp)
{
    __shared__ uint32_t hist[kBins1];
    __shared__ __attribute__((aligned(16))) uint32_t wbins[kBinsW];
    __shared__ uint32_t verdict[6];              // found, bin, rest lo, rest hi, candidates lo, hi
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    // everything the verdict and its record need is asked for up front: one memory latency, not three in a row
    const uint32_t hint = *sc.hint, hint_shift = sc.hint[kHintShift], hint_hold = sc.hint[kHintHold], hint_cap = sc.hint[kHintCap];
    uint32_t open = wave == 0 ? sc.hist[kHistOpen + lane] : 0u;
    for (int b = t; b < kBinsW; b += kSeedThreads) {          // the window: the sum of its copies
        uint32_t sum = 0;
#pragma unroll
        for (int r = 0; r < kWinCopies; ++r) sum += sc.hist[kHistW + r * kBinsW + b];
        wbins[b] = sum;
    }
    __syncthreads();
    if (wave == 0) {
        uint32_t bin;
        uint64_t rest;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) open += __shfl_xor(open, d, 64);
        uint64_t cands;
        const bool found = resolve_lds<kBinsW>(wbins, k, bin, rest, open, &cands);
        if (lane == 0) {
            verdict[0] = found; verdict[1] = bin; verdict[2] = (uint32_t)rest; verdict[3] = (uint32_t)(rest >> 32);
            verdict[4] = (uint32_t)cands; verdict[5] = (uint32_t)(cands >> 32);
        }
    }
    for (int b = t; b < kBins1; b += kSeedThreads) hist[b] = 0u;
    __syncthreads();
    const bool found = verdict[0] != 0u;
    const uint32_t bin = verdict[1];
    if (found && bin < (uint32_t)kBinsW - 1u) {
        if (blockIdx.x == 0 && t == 0) {
            SelectState s;
            s.lo = hint + (bin << kWindowShift); s.mode = kModeFast; s.need = (uint64_t)verdict[2] | ((uint64_t)verdict[3] << 32);
            sc.sel[0] = s;
            margin_after_hit(sc.hint, hint_shift, hint_hold, hint_cap, (uint64_t)verdict[4] | ((uint64_t)verdict[5] << 32), k);
        }
        return;
    }
    // missed: the next calls filter with the full margin again, and keep it for a while
    if (blockIdx.x == 0 && t == 0) margin_after_miss(sc.hint, hint_shift, !found);
    const uint32_t ntiles = (g.n + (uint32_t)kTile - 1u) / (uint32_t)kTile;
    const uint32_t uwave = __builtin_amdgcn_readfirstlane(wave), waves = kSeedThreads / 64;
    if (found) {
        // ---- above the window
        const uint32_t lo = hint + (((uint32_t)kBinsW - 1u) << kWindowShift);
        for (uint32_t tile = blockIdx.x * waves + uwave; tile < ntiles; tile += gridDim.x * waves) {
            tile_walk<true>(sc, tile, sc.tile_runs[tile], [&](bool valid, uint32_t chunk, uint32_t bits, uint32_t loc) {
                const uint32_t key = bits & 0x7FFFFFFFu;
                if (valid && key >= lo && in_sample(smp, chunk * (uint32_t)kChunk + loc)) atomicAdd(&hist[(key - lo) >> 20], 1u);
            });
        }
        __syncthreads();
        flush_fine(hist, sc.hist + kHist1, kBins1);
        if (blockIdx.x == 0 && t == 0) {
            SelectState s;
            s.lo = lo; s.mode = 0u; s.need = k;
            sc.sel[0] = s;
        }
        return;
    }
    // ---- refill
    const uint32_t nch = (g.n + (uint32_t)kChunk - 1u) / (uint32_t)kChunk;
    for (uint32_t ch = blockIdx.x * waves + uwave; ch < nch; ch += gridDim.x * waves) {
        Chunk c;
        c.base = ch * (uint32_t)kChunk;
        c.lane = lane;
        c.full = g.n - c.base >= (uint32_t)kChunk;
        uint32_t bits[kSteps];
        if (RANDOM) {
            chunk_words(rng.seed, rng.worker, rng.iter_lo, g.goff + c.base, c.lane, bits);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) bits[j] >>= 1;
        } else {
            float v[kSteps];
            load_sel<FROM_STATE>(g, st, c, v);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) bits[j] = __float_as_uint(v[j]);
        }
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            uint32_t i = c.base + 64 * j + c.lane;
            if (c.full || i < g.n) {
                sc.cand_bits[i] = bits[j];
                sc.cand_loc[i] = (uint16_t)(64 * j + c.lane);
                if (in_sample(smp, i)) atomicAdd(&hist[(bits[j] & 0x7FFFFFFFu) >> 20], 1u);
            }
        }
    }
    __syncthreads();
    flush_fine(hist, sc.hist + kHist1, kBins1);
    if (blockIdx.x == 0 && t == 0) {
        SelectState s;
        s.lo = 0u; s.mode = kModeUniform; s.need = k;
        sc.sel[0] = s;
    }
}

// ---------------------------------------------------------------------------
// level 2 / level 3 histogram over the candidates, one tile per wavefront
//   LEVEL 2: nothing to do after a fast seed.  Otherwise resolves level 1 (2048 bins of
//            2^20 keys above the seed's lo) and histograms bits 19..10 of key - lo
//   LEVEL 3: after a fast seed lo / need come from the seed; otherwise resolves level 2.
//            Histograms the last 10 bits
// Block 0 records the resolved state for the next kernel and clears the histogram
// that the previous kernel has finished reading.
// ---------------------------------------------------------------------------
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void cand_hist_k(uint32_t n, uint32_t ntiles, SparseScratch sc, SampleRule smp)
{
    constexpr int kBins = LEVEL == 2 ? kBins2 : kBins3;
    __shared__ uint32_t hist[kBins];
    const SelectState s0 = sc.sel[0];
    if (LEVEL == 2) {
        // the seed is done with the window: all blocks clear it together (one block alone is the whole duration of
        // this kernel on the fast route: 1.5 us)
        for (uint32_t b = blockIdx.x * kBlock + threadIdx.x; b < (uint32_t)(kWinCopies * kBinsW + kOpenCopies); b += gridDim.x * kBlock)
            sc.hist[b < (uint32_t)(kWinCopies * kBinsW) ? kHistW + b : kHistOpen - kWinCopies * kBinsW + b] = 0u;
        if (s0.mode & kModeFast) return;
    }
    const bool uniform = (s0.mode & kModeUniform) != 0u;
    TileJob job = my_tile(sc, n, ntiles);
    for (int b = threadIdx.x; b < kBins; b += kBlock) hist[b] = 0u;
    uint32_t lo;
    uint64_t need;
    if (LEVEL == 2) {
        uint32_t bin;
        resolve_wave<kBins1>(sc.hist + kHist1, s0.need, bin, need);
        lo = s0.lo + (bin << 20);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            SelectState s;
            s.lo = lo; s.mode = s0.mode; s.need = need;
            sc.sel[1] = s;
        }
    } else {
        if (s0.mode & kModeFast) { lo = s0.lo; need = s0.need; }
        else {
            const SelectState s1 = sc.sel[1];
            uint32_t bin;
            resolve_wave<kBins2>(sc.hist + kHist2, s1.need, bin, need);
            lo = s1.lo + (bin << 10);
        }
        if (blockIdx.x == 0) {
            if (threadIdx.x == 0) {
                SelectState s;
                s.lo = lo; s.mode = s0.mode; s.need = need;
                sc.sel[2] = s;
            }
            for (int b = threadIdx.x; b < kBins1; b += kBlock) sc.hist[kHist1 + b] = 0u;   // level 2 is done with level 1
        }
    }
    __syncthreads();
    if (uniform) job.runs = job.tile < ntiles ? uniform_runs(job.tile, n) : 0ull;
    // keys still undecided: level 2 leaves 2^10 to level 3; a fast seed leaves a whole window bin
    const uint32_t kRange = LEVEL == 2 ? 1u << 20 : (s0.mode & kModeFast) ? 1u << kWindowShift : 1u << 10;
    constexpr int kShift = LEVEL == 2 ? 10 : 0;
    uint32_t any = 0;
    tile_walk<true>(sc, job.tile, job.runs, [&](bool valid, uint32_t chunk, uint32_t bits, uint32_t loc) {
        const uint32_t d = (bits & 0x7FFFFFFFu) - lo;       // wraps to a large number for keys below lo
        if (valid && d < kRange && in_sample(smp, chunk * (uint32_t)kChunk + loc)) { atomicAdd(&hist[d >> kShift], 1u); any = 1u; }
    });
    if (__syncthreads_or((int)any)) flush_fine(hist, sc.hist + (LEVEL == 2 ? kHist2 : kHist3), kBins);
}

// ---------------------------------------------------------------------------
// count: resolve level 3 -> threshold key T and `need` (keys == T to take, in
// index order); candidates above / equal to T per tile and per block of four tiles.
// ---------------------------------------------------------------------------
// (six wavefronts per SIMD hold all tiles of the ResNet-50 buffer at once; left alone the compiler takes 102 registers: four)
__attribute__((amdgpu_waves_per_eu(6, 6)))
__global__ __launch_bounds__(kBlock) void cand_count_k(uint32_t n, uint32_t ntiles, SparseScratch sc)
{
    __shared__ uint32_t wgt[kWavesPerBlock], weq[kWavesPerBlock];
    __shared__ uint32_t res[3];
    TileJob job = my_tile(sc, n, ntiles);
    const SelectState s2 = sc.sel[2];
    const uint32_t hint_shift = sc.hint[kHintShift];        // (asked for now: block 0 would wait for it later)
    // one wavefront reads the bins for the block: every wavefront doing so would move the histogram
    // once per tile of the group
    if (threadIdx.x < 64) {
        uint32_t b;
        uint64_t r;
        resolve_wave<kBins3>(sc.hist + kHist3, s2.need, b, r);
        if (threadIdx.x == 0) { res[0] = b; res[1] = (uint32_t)r; res[2] = (uint32_t)(r >> 32); }
    }
    __syncthreads();
    const uint32_t bin = res[0];
    const uint64_t rest = (uint64_t)res[1] | ((uint64_t)res[2] << 32);
    const uint32_t T = s2.lo + bin;
    if (blockIdx.x == 0) {
        if (threadIdx.x == 0) {
            SelectState s;
            s.lo = T; s.mode = s2.mode; s.need = rest;
            sc.sel[3] = s;
            const uint32_t margin = kHintMargin >> hint_shift;
            *sc.hint = T > margin ? T - margin : 0u;                // where the next call starts filtering
        }
        for (int b = threadIdx.x; b < kBins2; b += kBlock) sc.hist[kHist2 + b] = 0u;   // level 3 is done with level 2
    }
    if (s2.mode & kModeUniform) job.runs = job.tile < ntiles ? uniform_runs(job.tile, n) : 0ull;
    uint32_t ngt = 0, neq = 0;
    tile_walk<false>(sc, job.tile, job.runs, [&](bool valid, uint32_t, uint32_t bits, uint32_t) {
        uint32_t key = bits & 0x7FFFFFFFu;
        ngt += __popcll(__builtin_amdgcn_ballot_w64(valid && key > T));
        neq += __popcll(__builtin_amdgcn_ballot_w64(valid && key == T));
    });
    const uint32_t wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63u) == 0) {
        wgt[wave] = ngt; weq[wave] = neq;
        if (job.tile < ntiles) sc.tile_cnt[job.tile] = ngt | (neq << 16);     // a tile holds at most 4096 candidates
    }
    __syncthreads();
    if (threadIdx.x == 0)                                                      // a block at most 16384
        sc.blk_cnt[blockIdx.x] = (wgt[0] + wgt[1] + wgt[2] + wgt[3]) | ((weq[0] + weq[1] + weq[2] + weq[3]) << 16);
}

// ---------------------------------------------------------------------------
// emit: ordered compaction.  A candidate is kept if its key is above T, or equal
// to T and among the first `need` such keys in index order.  Its slot is
//   (#kept before it) = (#above before it) + min(#equal before it, need).
// Every block adds up the counts of the blocks before it; nothing waits.
// ---------------------------------------------------------------------------
// The directory that ends a sparse payload: entry t = kept entries with index below 4096 t, t = 0 .. tiles (the paper
// gives no payload format; this one lets the receiver find a payload's share of a tile without searching).  It follows
// the index and value lists, which have room for `cap` entries each.
__device__ __forceinline__ uint32_t *payload_directory(PayloadHeader *hdr, uint64_t cap)
{
    return reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(hdr) + kHeaderBytes + 8u * cap);
}

// What the compaction does to the memory of an entry it keeps.  Top-k and DGC leave entries above the threshold key to the
// next call's streaming pass (StateHeader::sent_key) and zero only kept entries equal to it; Rand-k, whose choice does not
// depend on the values, zeroes in place.
template <int ALGO, bool EF>
__device__ __forceinline__ void drop_sent(float *st, uint32_t n, uint32_t i, bool equal)
{
    if (ALGO == MC_ALGO_RANDK) st[i] = 0.0f;
    else if (ALGO == MC_ALGO_DGC) { if (equal) { st[i] = 0.0f; st[dgc_u_offset(n) + i] = 0.0f; } }      // momentum factor masking
    else if (EF) { if (equal) st[i] = 0.0f; }
}
// ... and what it tells the next call (one thread)
template <int ALGO, bool EF>
__device__ __forceinline__ void record_sent_key(float *st, uint32_t T)
{
    if (ALGO == MC_ALGO_DGC || EF)
        reinterpret_cast<StateHeader *>(reinterpret_cast<uint8_t *>(st) - kHeaderBytes)->sent_key = ALGO == MC_ALGO_RANDK ? 0xFFFFFFFFu : T;
}

// The walk of one tile's candidates that both emit kernels share: gt_before / eq_before are the numbers of keys
// above / equal to T among all candidates before this tile.
template <int ALGO, bool EF>
__device__ __forceinline__ void emit_tile(const SparseScratch &sc, uint32_t tile, uint64_t runs, uint32_t n, uint64_t k, float *st,
                                          uint32_t *idx, float *val, uint32_t T, uint64_t need, uint64_t gt_before, uint64_t eq_before)
{
    tile_walk<true>(sc, tile, runs, [&](bool valid, uint32_t chunk, uint32_t b, uint32_t loc) {
        const uint32_t key = b & 0x7FFFFFFFu;
        const bool is_gt = valid && key > T, is_eq = valid && key == T;
        const uint64_t bgt = __builtin_amdgcn_ballot_w64(is_gt), beq = __builtin_amdgcn_ballot_w64(is_eq);
        const uint64_t gtb = gt_before + lanes_below(bgt), eqb = eq_before + lanes_below(beq);
        if (is_gt || (is_eq && eqb < need)) {
            const uint64_t pos = gtb + (eqb < need ? eqb : need);
            const uint32_t i = chunk * (uint32_t)kChunk + loc;
            if (pos < k && i < n) {                  // exact selection: always true for consistent scratch; CAPPED: room left
                idx[pos] = i;
                if (ALGO == MC_ALGO_RANDK) val[pos] = st[i];      // the candidate slot holds the random key: the value is p
                else val[pos] = __uint_as_float(b);
                if (ALGO == MC_ALGO_DGC) { st[i] = 0.0f; st[dgc_u_offset(n) + i] = 0.0f; }   // momentum factor masking
                else if (EF) st[i] = 0.0f;
            }
        }
        gt_before += __popcll(bgt);
        eq_before += __popcll(beq);
    });
}

// CAPPED (DGC with a sampled threshold): T comes from the sample, so the number of keys >= T varies.
// k is then the payload's capacity: all keys above T are kept in index order while there is room, then
// keys equal to T; the header records how many entries were kept and unused entries are zeroed.
template <int ALGO, bool EF, bool CAPPED>
__global__ __launch_bounds__(kBlock) void cand_emit_k(uint32_t n, uint32_t ntiles, float *st, PayloadHeader *hdr, uint64_t k,
                                                      SparseScratch sc)
{
    __shared__ uint64_t sgt[kWavesPerBlock], seq[kWavesPerBlock], stg[kWavesPerBlock], ste[kWavesPerBlock];
    TileJob job = my_tile(sc, n, ntiles);
    const SelectState s3 = sc.sel[3];
    const uint32_t T = s3.lo;
    uint64_t need = s3.need;
    uint32_t *idx = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(hdr) + kHeaderBytes);
    float *val = reinterpret_cast<float *>(idx + k);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    // kept-before of this wavefront inside the block
    uint64_t wg = 0, we = 0;
    if (lane < wave && job.tile < ntiles) {          // then the tiles before it in the block exist too
        const uint32_t x = sc.tile_cnt[blockIdx.x * kWavesPerBlock + lane];
        wg = x & 0xFFFFu; we = x >> 16;
    }
    // kept-before of this block: sum over the blocks before it (CAPPED: and over all blocks), eight loads in
    // flight per thread
    uint64_t ag = 0, ae = 0, tg = 0, te = 0;
    const uint32_t upto = CAPPED ? gridDim.x : blockIdx.x;
    for (uint32_t b0 = 0; b0 < upto; b0 += 8 * kBlock) {
        uint32_t x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t b = b0 + u * kBlock + threadIdx.x;
            x[u] = b < upto ? sc.blk_cnt[b] : 0u;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t b = b0 + u * kBlock + threadIdx.x;
            if (b < blockIdx.x) { ag += x[u] & 0xFFFFu; ae += x[u] >> 16; }
            if (CAPPED) { tg += x[u] & 0xFFFFu; te += x[u] >> 16; }
        }
    }
    if (blockIdx.x == 0)
        for (int b = threadIdx.x; b < kBins3; b += kBlock) sc.hist[kHist3 + b] = 0u;   // count is done with level 3
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        ag += __shfl_xor(ag, m, 64); ae += __shfl_xor(ae, m, 64);
        wg += __shfl_xor(wg, m, 64); we += __shfl_xor(we, m, 64);
        if (CAPPED) { tg += __shfl_xor(tg, m, 64); te += __shfl_xor(te, m, 64); }
    }
    if (lane == 0) { sgt[wave] = ag; seq[wave] = ae; stg[wave] = tg; ste[wave] = te; }
    __syncthreads();
    uint64_t gt_before = (sgt[0] + sgt[1]) + (sgt[2] + sgt[3]) + wg;
    uint64_t eq_before = (seq[0] + seq[1]) + (seq[2] + seq[3]) + we;
    uint64_t kept = k;
    if (CAPPED) {
        const uint64_t all_gt = (stg[0] + stg[1]) + (stg[2] + stg[3]), all_eq = (ste[0] + ste[1]) + (ste[2] + ste[3]);
        const uint64_t kept_gt = all_gt < k ? all_gt : k;
        need = all_eq < k - kept_gt ? all_eq : k - kept_gt;
        kept = kept_gt + need;
        // entries of the payload that stay unused are zero
        for (uint64_t pos = kept + (uint64_t)blockIdx.x * kBlock + threadIdx.x; pos < k; pos += (uint64_t)gridDim.x * kBlock) {
            idx[pos] = 0u;
            val[pos] = 0.0f;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        PayloadHeader h;
        h.magic = kMagic; h.algo = ALGO; h.n = n; h.k = kept; h.scale = 0.0f; h.levels = CAPPED ? (uint32_t)k : 0u;
        for (int i = 0; i < 24; ++i) h.pad[i] = 0;
        *hdr = h;
        // this kernel zeroes what it keeps in place: the next streaming pass has nothing to mask
        if (ALGO == MC_ALGO_DGC || EF) reinterpret_cast<StateHeader *>(reinterpret_cast<uint8_t *>(st) - kHeaderBytes)->sent_key = 0xFFFFFFFFu;
    }
    if (s3.mode & kModeUniform) job.runs = job.tile < ntiles ? uniform_runs(job.tile, n) : 0ull;
    if (lane == 0 && job.tile < ntiles) {
        uint32_t *dir = payload_directory(hdr, k);
        const uint64_t at = gt_before + (eq_before < need ? eq_before : need);      // CAPPED: there may be no room for all of them
        dir[job.tile] = (uint32_t)(at < kept ? at : kept);
        if (job.tile == ntiles - 1u) dir[ntiles] = (uint32_t)kept;
    }
    emit_tile<ALGO, EF>(sc, job.tile, job.runs, n, k, st, idx, val, T, need, gt_before, eq_before);
}

// ---------------------------------------------------------------------------
// The two-kernel tail (everything but DGC with a sampled threshold).
//
//   select   every block (16 wavefronts, one 4096-element tile each) resolves the window on its own -- no
//            kernel in between just to reduce 2048 bins -- and all blocks reach the same verdict:
//     lean     the threshold lies in window bin b, which holds at most kUCap keys.  Every key above the
//              bin is kept whatever the threshold turns out to be: their number per tile and per block is
//              all the emit kernel needs of them.  The keys inside the bin -- a few hundred out of
//              millions -- are appended to a list.
//     dense    bin b holds more than kUCap keys (heavy ties, or a pile of values just under the
//              threshold): the blocks histogram its 2048 keys, as level 3 of a radix select
//     above    the threshold lies above the window: level 1 (bits 30..20 above the window's top) over
//              the candidates
//     refill   fewer than k candidates: every element becomes a candidate, level 1 over all keys
//   emit     lean: every block reads the whole list (it is small), finds the threshold key T and the
//            number of keys equal to T to take with a histogram in LDS, counts the list's kept keys
//            that lie before each of its tiles, adds the kept counts of the blocks before it, and
//            compacts its tiles' kept candidates into the payload.  One kernel after the select: no
//            level-3 pass, no counting pass.
//            Otherwise the remaining radix levels, the per-tile counts and the compaction run as steps
//            of this same kernel on as many blocks as the device surely holds at once, separated by
//            grid-wide barriers: the rare routes cost no launch on the usual one.
// Both kernels are bound by memory latency, not by traffic, so each asks for its tile's candidates as soon
// as it knows how many there are, before it waits for anything else.
// ---------------------------------------------------------------------------
constexpr int kSelThreads = 1024, kSelWaves = kSelThreads / 64;      // select: 16 tiles per block (the window is read once per block)
constexpr int kEmitThreads = kBlock, kEmitWaves = kWavesPerBlock;    // emit: 4 tiles per block
constexpr int kSyncArrive = 0, kSyncRoutes = 32, kSyncLastBin = 40, kSyncLastCands = 41;     // words of SparseScratch::sync (mc_api.hip reads the last three)

struct TileRuns { uint32_t r0, r1, r2, total; };       // running sums of the candidates of a tile's four chunks
__device__ __forceinline__ TileRuns decode_runs(uint64_t runs)
{
    TileRuns r;
    r.r0 = (uint32_t)(runs & 0xFFFFu); r.r1 = r.r0 + (uint32_t)((runs >> 16) & 0xFFFFu);
    r.r2 = r.r1 + (uint32_t)((runs >> 32) & 0xFFFFu); r.total = r.r2 + (uint32_t)(runs >> 48);
    return r;
}

// ROUNDS rounds of 64 of a tile's candidates, from candidate number f0 on; candidate f0 + 64 u + lane is there if
// that number is below the tile's total.  at: group-relative index of the element.
template <int ROUNDS>
struct CandBatch { uint32_t bits[ROUNDS], at[ROUNDS]; };

template <int ROUNDS, bool WITH_AT>
__device__ __forceinline__ void fetch_batch(const SparseScratch &sc, uint32_t tile, const TileRuns &r, uint32_t f0, CandBatch<ROUNDS> &c)
{
    const uint32_t lane = threadIdx.x & 63u;
    size_t slot[ROUNDS];
    bool valid[ROUNDS];
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        const uint32_t f = f0 + 64 * u + lane;
        valid[u] = f < r.total;
        const uint32_t s = (f >= r.r0) + (f >= r.r1) + (f >= r.r2);          // chunk of the tile, then slot inside it
        const uint32_t off = f - (s == 0 ? 0u : s == 1 ? r.r0 : s == 2 ? r.r1 : r.r2);
        const uint32_t ch = tile * (uint32_t)kWavesPerBlock + (valid[u] ? s : 0u);
        slot[u] = valid[u] ? (size_t)ch * kChunk + off : (size_t)tile * kTile;
        c.at[u] = ch * (uint32_t)kChunk;
    }
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        c.bits[u] = 0u;
        if (valid[u]) {
            c.bits[u] = sc.cand_bits[slot[u]];
            if (WITH_AT) c.at[u] += sc.cand_loc[slot[u]];
        }
    }
}

// Walk of a tile's candidates, 64 ROUNDS at a time (the slow routes: one memory latency per batch, so a crowded
// tile wants large batches).  body(valid, bits, at).
template <bool WITH_AT, int ROUNDS, typename Body>
__device__ __forceinline__ void walk_small(const SparseScratch &sc, uint32_t tile, uint64_t runs, Body body)
{
    const TileRuns r = decode_runs(runs);
    const uint32_t lane = threadIdx.x & 63u;
    for (uint32_t f0 = 0; f0 < r.total; f0 += 64 * ROUNDS) {
        CandBatch<ROUNDS> c;
        fetch_batch<ROUNDS, WITH_AT>(sc, tile, r, f0, c);
#pragma unroll
        for (int u = 0; u < ROUNDS; ++u)
            if (f0 + 64 * u < r.total) body(f0 + 64 * u + lane < r.total, c.bits[u], c.at[u]);
    }
}
constexpr int kWalkRounds = 16, kCompactRounds = 8;      // candidates in flight per wavefront in the slow routes: 1024 when only read, 512 when placed

// Select.  The keys inside the threshold's bin [lo, lo + 2048) -- rarely more than a few per tile -- are collected
// in a buffer of the wavefront's own in LDS and appended to sublist `sub` with one atomic add per tile (per 64
// entries when there are more): an add per batch of candidates put its latency between the batches.
constexpr int kMemberBuf = 64;
struct MemberBuf { UEntry *buf; uint32_t held; };

__device__ __forceinline__ void flush_members(const SparseScratch &sc, MemberBuf &m, uint32_t sub)
{
    if (!m.held) return;
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(&sc.ucount[sub * kUCountStride], m.held);
    base = __builtin_amdgcn_readfirstlane(base);
    __builtin_amdgcn_wave_barrier();
    if (lane < m.held && base + lane < kUCap) sc.ulist[(size_t)sub * kUCap + base + lane] = m.buf[lane];   // (always in range: the bin holds at most kUCap keys)
    __builtin_amdgcn_wave_barrier();
    m.held = 0u;
}

// Emit, one batch: a candidate is kept if its key is above T, or equal to T and among the first `need` such keys in
// index order; its place in the payload is (keys above T before it) + min(keys equal to T before it, need).
template <int ALGO, bool EF, int ROUNDS>
__device__ __forceinline__ void emit_apply(const CandBatch<ROUNDS> &c, uint32_t total, uint32_t f0, uint32_t n, uint64_t k, float *st,
                                           uint32_t *idx, float *val, uint32_t T, uint64_t need, uint64_t &gt_before, uint64_t &eq_before)
{
    const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
    for (int u = 0; u < ROUNDS; ++u) {
        if (f0 + 64 * u >= total) break;
        const bool valid = f0 + 64 * u + lane < total;
        const uint32_t key = c.bits[u] & 0x7FFFFFFFu;
        const bool is_gt = valid && key > T, is_eq = valid && key == T;
        const uint64_t bgt = __builtin_amdgcn_ballot_w64(is_gt), beq = __builtin_amdgcn_ballot_w64(is_eq);
        const uint64_t gtb = gt_before + lanes_below(bgt), eqb = eq_before + lanes_below(beq);
        if (is_gt || (is_eq && eqb < need)) {
            const uint64_t pos = gtb + (eqb < need ? eqb : need);
            const uint32_t i = c.at[u];
            if (pos < k && i < n) {                  // always true for consistent scratch
                idx[pos] = i;
                if (ALGO == MC_ALGO_RANDK) val[pos] = st[i];      // the candidate slot holds the random key: the value is p
                else val[pos] = __uint_as_float(c.bits[u]);
                drop_sent<ALGO, EF>(st, n, i, is_eq);
            }
        }
        gt_before += __popcll(bgt);
        eq_before += __popcll(beq);
    }
}

__device__ __forceinline__ void put_sparse_header(PayloadHeader *hdr, uint32_t algo, uint32_t n, uint64_t k)
{
    PayloadHeader h;
    h.magic = kMagic; h.algo = algo; h.n = n; h.k = k; h.scale = 0.0f; h.levels = 0u;
    for (int i = 0; i < 24; ++i) h.pad[i] = 0;
    *hdr = h;
}
// where the next call of this (group, worker) starts filtering: a margin below this call's threshold key
__device__ __forceinline__ void publish_hint(const SparseScratch &sc, uint32_t T)
{
    const uint32_t margin = kHintMargin >> sc.hint[kHintShift];
    *sc.hint = T > margin ? T - margin : 0u;
}

// Grid-wide barrier of the slow routes, for the first `blocks` blocks of the grid, all of which the device
// holds at once (one per compute unit at most): arrivals are counted in one word (cleared by the streaming pass),
// the `round`-th barrier is passed when it reaches round * blocks.  The release / acquire pair makes what every
// block wrote before the barrier visible to every block after it.  The wait is bounded: should the count never
// come (it always does when the blocks are resident together), the block flags the failure and leaves, and so
// does every later wait.
__device__ __forceinline__ bool grid_barrier(uint32_t *arrive, uint32_t blocks, uint32_t round, uint32_t *dead /* LDS */, int *status, uint32_t limit)
{
    __syncthreads();
    if (threadIdx.x == 0 && !*dead) {
        __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t target = round * blocks;
        uint32_t spins = 0;
        // polled without acquire semantics: an acquire at agent scope invalidates the die's L2, and two hundred waiting
        // blocks doing that every few hundred cycles starve the blocks still at work (phases of 60-120 us instead of 10)
        while (__hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(32);
            if (spins++ >= limit) { *dead = 1u; *status = 2; break; }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
    return *dead == 0u;
}

// a radix level resolved for the whole block by its first wavefront
template <int BINS>
__device__ __forceinline__ void resolve_block(const uint32_t *fine, uint64_t need, uint32_t &bin, uint64_t &rest, uint32_t *res /* 3 words of LDS */)
{
    if (threadIdx.x < 64) {
        uint32_t b;
        uint64_t r;
        resolve_wave<BINS>(fine, need, b, r);
        if (threadIdx.x == 0) { res[0] = b; res[1] = (uint32_t)r; res[2] = (uint32_t)(r >> 32); }
    }
    __syncthreads();
    bin = res[0];
    rest = (uint64_t)res[1] | ((uint64_t)res[2] << 32);
    __syncthreads();
}

constexpr int kRoundTiles = 4096;      // tiles per round of the slow routes' compaction: 256 blocks of 16 wavefronts at most

// The routes that need more than the window: all radix levels still open, the per-tile counts and the ordered
// compaction, as steps of one kernel of `blocks` blocks (which the device holds at once), each
// wavefront taking tiles gw, gw + nw, ...  `mode`: what the window said (kModeFast | kModeDense: the threshold's
// bin [lo, lo + 2048) is known but too full to list; 0: the threshold lies above lo, the window's top;
// kModeUniform: too few candidates, every element becomes one).
template <int ALGO, bool EF, bool FROM_STATE, bool RANDOM>
__device__ __forceinline__ void slow_routes(const GroupView &g, float *st, PayloadHeader *hdr, uint64_t k, const SparseScratch &sc,
                                            const RngKey &rng, uint32_t mode, uint32_t lo, uint64_t need, uint32_t blocks, int *status,
                                            uint32_t *hist /* 2048 words of LDS */, uint32_t *pfx /* 2 * kRoundTiles words of LDS */,
                                            uint32_t *small /* 64 words of LDS */)
{
    uint32_t *res = small, *dead = small + 4, *wsum = small + 8;      // wsum: 2 * kSelWaves words
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const uint32_t n = g.n, ntiles = (n + (uint32_t)kTile - 1u) / (uint32_t)kTile;
    const uint32_t nw = blocks * kSelWaves, gw = blockIdx.x * kSelWaves + wave;
    const bool uniform = (mode & kModeUniform) != 0u;
    if (t == 0) *dead = 0u;
    uint32_t round = 0, T, bin;
    auto runs_of = [&](uint32_t tile) { return uniform ? uniform_runs(tile, n) : sc.tile_runs[tile]; };
    for (int b = t; b < kBins1; b += kSelThreads) hist[b] = 0u;
    __syncthreads();
    if (!(mode & kModeFast)) {
        // ---- level 1: bits 30..20 of key - lo
        if (!uniform) {
            for (uint32_t tile = gw; tile < ntiles; tile += nw)
                walk_small<false, kWalkRounds>(sc, tile, runs_of(tile), [&](bool valid, uint32_t bits, uint32_t) {
                    const uint32_t key = bits & 0x7FFFFFFFu;
                    if (valid && key >= lo) atomicAdd(&hist[(key - lo) >> 20], 1u);
                });
        } else {
            // refill: every element becomes a candidate (chunk c holds candidates 1024 c ...)
            const uint32_t nch = (n + (uint32_t)kChunk - 1u) / (uint32_t)kChunk;
            for (uint32_t ch = gw; ch < nch; ch += nw) {
                Chunk c;
                c.base = ch * (uint32_t)kChunk;
                c.lane = lane;
                c.full = n - c.base >= (uint32_t)kChunk;
                uint32_t bits[kSteps];
                if (RANDOM) {
                    chunk_words(rng.seed, rng.worker, rng.iter_lo, g.goff + c.base, c.lane, bits);
#pragma unroll
                    for (int j = 0; j < kSteps; ++j) bits[j] >>= 1;
                } else {
                    float v[kSteps];
                    load_sel<FROM_STATE>(g, st, c, v);
#pragma unroll
                    for (int j = 0; j < kSteps; ++j) bits[j] = __float_as_uint(v[j]);
                }
#pragma unroll
                for (int j = 0; j < kSteps; ++j) {
                    const uint32_t i = c.base + 64 * j + c.lane;
                    if (c.full || i < n) {
                        sc.cand_bits[i] = bits[j];
                        sc.cand_loc[i] = (uint16_t)(64 * j + c.lane);
                        atomicAdd(&hist[(bits[j] & 0x7FFFFFFFu) >> 20], 1u);
                    }
                }
            }
        }
        __syncthreads();
        flush_fine(hist, sc.hist + kHist1, kBins1);
        if (!grid_barrier(sc.sync + kSyncArrive, blocks, ++round, dead, status, sc.spin_limit)) return;
        resolve_block<kBins1>(sc.hist + kHist1, need, bin, need, res);
        lo += bin << 20;
        // ---- level 2: bits 19..10
        for (int b = t; b < kBins2; b += kSelThreads) hist[b] = 0u;
        __syncthreads();
        for (uint32_t tile = gw; tile < ntiles; tile += nw)
            walk_small<false, kWalkRounds>(sc, tile, runs_of(tile), [&](bool valid, uint32_t bits, uint32_t) {
                const uint32_t key = bits & 0x7FFFFFFFu;
                if (valid && key >= lo && key - lo < (1u << 20)) atomicAdd(&hist[(key - lo) >> 10], 1u);
            });
        __syncthreads();
        flush_fine(hist, sc.hist + kHist2, kBins2);
        if (!grid_barrier(sc.sync + kSyncArrive, blocks, ++round, dead, status, sc.spin_limit)) return;
        if (blockIdx.x == 0) for (int b = t; b < kBins1; b += kSelThreads) sc.hist[kHist1 + b] = 0u;    // every block has resolved level 1
        resolve_block<kBins2>(sc.hist + kHist2, need, bin, need, res);
        lo += bin << 10;
        for (int b = t; b < kBins3; b += kSelThreads) hist[b] = 0u;
        __syncthreads();
    }
    // ---- level 3: the bits still open (10 after level 2, the 11 of a window bin otherwise)
    const uint32_t open = (mode & kModeFast) ? 1u << kWindowShift : 1u << 10;
    for (uint32_t tile = gw; tile < ntiles; tile += nw)
        walk_small<false, kWalkRounds>(sc, tile, runs_of(tile), [&](bool valid, uint32_t bits, uint32_t) {
            const uint32_t key = bits & 0x7FFFFFFFu;
            if (valid && key >= lo && key - lo < open) atomicAdd(&hist[key - lo], 1u);
        });
    __syncthreads();
    flush_fine(hist, sc.hist + kHist3, kBins3);
    if (!grid_barrier(sc.sync + kSyncArrive, blocks, ++round, dead, status, sc.spin_limit)) return;
    if (!(mode & kModeFast) && blockIdx.x == 0) for (int b = t; b < kBins2; b += kSelThreads) sc.hist[kHist2 + b] = 0u;
    resolve_block<kBins3>(sc.hist + kHist3, need, bin, need, res);
    T = lo + bin;
    // ---- kept candidates per tile
    for (uint32_t tile = gw; tile < ntiles; tile += nw) {
        uint32_t ngt = 0, neq = 0;
        walk_small<false, kWalkRounds>(sc, tile, runs_of(tile), [&](bool valid, uint32_t bits, uint32_t) {
            const uint32_t key = bits & 0x7FFFFFFFu;
            ngt += __popcll(__builtin_amdgcn_ballot_w64(valid && key > T));
            neq += __popcll(__builtin_amdgcn_ballot_w64(valid && key == T));
        });
        if (lane == 0) sc.tile_cnt[tile] = ngt | (neq << 16);              // a tile holds at most 4096 candidates
    }
    if (!grid_barrier(sc.sync + kSyncArrive, blocks, ++round, dead, status, sc.spin_limit)) return;
    if (blockIdx.x == 0) for (int b = t; b < kBins3; b += kSelThreads) sc.hist[kHist3 + b] = 0u;
    uint32_t *idx = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(hdr) + kHeaderBytes);
    float *val = reinterpret_cast<float *>(idx + k);
    if (blockIdx.x == 0 && t == 0) {
        put_sparse_header(hdr, ALGO, n, k);
        SelectState s;
        s.lo = T; s.mode = mode; s.need = need;
        sc.sel[3] = s;
        publish_hint(sc, T);
        record_sent_key<ALGO, EF>(st, T);
    }
    // ---- ordered compaction, kRoundTiles tiles at a time: every block scans the round's counts (in LDS) for the
    // keys kept before each tile, and carries the totals of the rounds before
    uint64_t base_gt = 0, base_eq = 0;
    constexpr int kPer = kRoundTiles / kSelThreads;
    for (uint32_t r0 = 0; r0 < ntiles; r0 += kRoundTiles) {
        uint32_t cg[kPer], ce[kPer], sg = 0, se = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const uint32_t tile = r0 + t * kPer + i;
            const uint32_t x = tile < ntiles ? sc.tile_cnt[tile] : 0u;
            cg[i] = x & 0xFFFFu; ce[i] = x >> 16;
            sg += cg[i]; se += ce[i];
        }
        uint32_t ig = sg, ie = se;                                          // inclusive scan over the block's threads
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t og = __shfl_up(ig, d, 64), oe = __shfl_up(ie, d, 64);
            if (lane >= (uint32_t)d) { ig += og; ie += oe; }
        }
        if (lane == 63u) { wsum[wave] = ig; wsum[kSelWaves + wave] = ie; }
        __syncthreads();
        uint32_t wg = 0, we = 0, tg = 0, te = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {
            if ((uint32_t)w < wave) { wg += wsum[w]; we += wsum[kSelWaves + w]; }
            tg += wsum[w]; te += wsum[kSelWaves + w];
        }
        uint32_t xg = wg + ig - sg, xe = we + ie - se;                       // kept before this thread's first tile, inside the round
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            pfx[t * kPer + i] = xg; pfx[kRoundTiles + t * kPer + i] = xe;
            xg += cg[i]; xe += ce[i];
        }
        __syncthreads();
        for (uint32_t p = gw; p < (uint32_t)kRoundTiles && r0 + p < ntiles; p += nw) {
            const uint32_t tile = r0 + p;
            const TileRuns tr = decode_runs(runs_of(tile));
            uint64_t gtb = base_gt + pfx[p], eqb = base_eq + pfx[kRoundTiles + p];
            if (lane == 0) {
                uint32_t *dir = payload_directory(hdr, k);
                dir[tile] = (uint32_t)(gtb + (eqb < need ? eqb : need));
                if (tile == ntiles - 1u) dir[ntiles] = (uint32_t)k;
            }
            for (uint32_t f0 = 0; f0 < tr.total; f0 += 64 * kCompactRounds) {
                CandBatch<kCompactRounds> c;
                fetch_batch<kCompactRounds, true>(sc, tile, tr, f0, c);
                emit_apply<ALGO, EF, kCompactRounds>(c, tr.total, f0, n, k, st, idx, val, T, need, gtb, eqb);
            }
        }
        base_gt += tg; base_eq += te;
        __syncthreads();
    }
}

// ---- access to the candidate slots of a tile ---------------------------------------------------------------
// A chunk's candidates sit at the front of its 1024 slots, in index order.  They are read as a *head* -- the first
// 64, one per lane -- and up to four *units* of 256 -- a lane takes four consecutive candidates with one 16-byte
// load of values and one 8-byte load of positions.  The kernels below live on memory latency, not on traffic: the
// heads of a tile's four chunks are asked for before the number of candidates is known (what lies beyond it is
// masked out afterwards; most chunks hold fewer than 64), and a crowded chunk costs one more round of loads, not
// one per 64 candidates.  Candidate number o >= 64 of a chunk is held by lane ((o - 64) % 256) / 4 of unit (o - 64) / 256.
constexpr int kHead = 64, kUnit = 256;
__device__ __forceinline__ uint32_t load_head_bits(const SparseScratch &sc, uint32_t chunk)
{
    return sc.cand_bits[(size_t)chunk * kChunk + (threadIdx.x & 63u)];
}
__device__ __forceinline__ uint32_t load_head_loc(const SparseScratch &sc, uint32_t chunk)
{
    return sc.cand_loc[(size_t)chunk * kChunk + (threadIdx.x & 63u)];
}
__device__ __forceinline__ uint4 load_bits4(const SparseScratch &sc, uint32_t chunk, uint32_t v)
{
    return *reinterpret_cast<const uint4 *>(sc.cand_bits + (size_t)chunk * kChunk + kHead + v * kUnit + (threadIdx.x & 63u) * 4u);
}
__device__ __forceinline__ uint2 load_loc4(const SparseScratch &sc, uint32_t chunk, uint32_t v)
{
    return *reinterpret_cast<const uint2 *>(sc.cand_loc + (size_t)chunk * kChunk + kHead + v * kUnit + (threadIdx.x & 63u) * 4u);
}
// x[q] for a q that is only known at run time, without putting the array into scratch memory
__device__ __forceinline__ uint32_t pick4(const uint32_t (&x)[4], uint32_t q) { return q == 0 ? x[0] : q == 1 ? x[1] : q == 2 ? x[2] : x[3]; }
__device__ __forceinline__ uint32_t elem4(const uint4 &x, int j) { return j == 0 ? x.x : j == 1 ? x.y : j == 2 ? x.z : x.w; }
__device__ __forceinline__ uint32_t loc4(const uint2 &x, int j) { return ((j < 2 ? x.x : x.y) >> (16 * (j & 1))) & 0xFFFFu; }
// is candidate (unit v, lane, j) of a chunk with cnt candidates there?
__device__ __forceinline__ bool in_unit(uint32_t cnt, uint32_t v, int j) { return (uint32_t)kHead + v * (uint32_t)kUnit + 4u * (threadIdx.x & 63u) + (uint32_t)j < cnt; }

// The units of a tile, numbered in chunk order: unit e is unit v of chunk q.
struct TileUnits {
    uint32_t per[kWavesPerBlock], total;
    __device__ __forceinline__ TileUnits(const uint32_t (&cnt)[kWavesPerBlock])
    {
        total = 0;
#pragma unroll
        for (int q = 0; q < kWavesPerBlock; ++q) { per[q] = cnt[q] > (uint32_t)kHead ? (cnt[q] - (uint32_t)kHead + (uint32_t)kUnit - 1u) / (uint32_t)kUnit : 0u; total += per[q]; }
    }
    __device__ __forceinline__ void locate(uint32_t e, uint32_t &q, uint32_t &v) const
    {
        q = 0;
#pragma unroll
        for (int i = 0; i < kWavesPerBlock - 1; ++i) if (q == (uint32_t)i && e >= per[i]) { e -= per[i]; ++q; }
        v = e;
    }
};

// Select: counts the keys above the threshold's bin, buffers those inside it (with the tile's first index: all that
// the emit kernel needs of a listed key's position is its tile).
__device__ __forceinline__ uint32_t select_one(const SparseScratch &sc, uint32_t bits, bool valid, uint32_t tile, uint32_t lo, uint32_t sub,
                                               MemberBuf &m)
{
    const uint32_t key = bits & 0x7FFFFFFFu;
    const bool reach = valid && key >= lo;
    const bool inside = reach && key - lo < (1u << kWindowShift);
    const uint64_t mb = __builtin_amdgcn_ballot_w64(inside);
    if (mb) {
        const uint32_t c = __popcll(mb);
        if (m.held + c > (uint32_t)kMemberBuf) flush_members(sc, m, sub);
        if (inside) { UEntry e; e.idx = tile * (uint32_t)kTile; e.bits = bits; m.buf[m.held + lanes_below(mb)] = e; }
        m.held += c;
    }
    return __popcll(__builtin_amdgcn_ballot_w64(reach && key - lo >= (1u << kWindowShift)));
}

// What a wavefront of the select kernel asks for of one tile before it knows the verdict.
struct TileAhead {
    uint32_t tile, cnt[kWavesPerBlock], head[kWavesPerBlock], uq[4], uv[4], units;
    uint4 ub[4];
};
__device__ __forceinline__ void look_ahead(const SparseScratch &sc, uint32_t tile, bool live, TileAhead &a)
{
    a.tile = tile;
    const uint64_t runs = live ? sc.tile_runs[tile] : 0ull;
    // the first 64 slots of each chunk, without waiting for the counts
#pragma unroll
    for (int q = 0; q < kWavesPerBlock; ++q) a.head[q] = live ? load_head_bits(sc, tile * kWavesPerBlock + q) : 0u;
    // ... and, as soon as the counts are there, the first four units of a tile with crowded chunks (nearly always all it has)
#pragma unroll
    for (int q = 0; q < kWavesPerBlock; ++q) a.cnt[q] = (uint32_t)(runs >> (16 * q)) & 0xFFFFu;
    const TileUnits tu(a.cnt);
    a.units = tu.total;
    if (tu.total) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            tu.locate((uint32_t)i < tu.total ? (uint32_t)i : 0u, a.uq[i], a.uv[i]);
            a.ub[i] = load_bits4(sc, tile * kWavesPerBlock + a.uq[i], a.uv[i]);
        }
    }
}
// ... and what it does with it on the lean route: the tile's keys above the threshold's bin are counted, those inside listed
__device__ __forceinline__ uint32_t select_tile(const SparseScratch &sc, TileAhead &a, uint32_t lo, uint32_t sub, MemberBuf &mb)
{
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t above = 0;
#pragma unroll
    for (int q = 0; q < kWavesPerBlock; ++q) if (a.cnt[q]) above += select_one(sc, a.head[q], lane < a.cnt[q], a.tile, lo, sub, mb);
    if (a.units) {
        const TileUnits tu(a.cnt);
        for (uint32_t e0 = 0; e0 < tu.total; e0 += 4u) {
            if (e0) {                            // (more than four units: the next four)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    tu.locate(e0 + i < tu.total ? e0 + i : e0, a.uq[i], a.uv[i]);
                    a.ub[i] = load_bits4(sc, a.tile * kWavesPerBlock + a.uq[i], a.uv[i]);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (e0 + i >= tu.total) break;
#pragma unroll
                for (int j = 0; j < 4; ++j) above += select_one(sc, elem4(a.ub[i], j), in_unit(pick4(a.cnt, a.uq[i]), a.uv[i], j), a.tile, lo, sub, mb);
            }
        }
    }
    if (lane == 0) sc.tile_cnt[a.tile] = above;
    return above;
}

// The select kernel: sixteen tiles per block, one wavefront each; the window is read once per block.
__global__ __launch_bounds__(kSelThreads) void lean_select_k(GroupView g, uint64_t k, SparseScratch sc)
{
    __shared__ uint32_t wtot[kSelWaves];
    __shared__ uint32_t verdict[8];              // found, bin, rest lo, rest hi, candidates lo, hi, keys in the bin
    __shared__ UEntry members[kSelWaves][kMemberBuf];
    __shared__ uint32_t wabove[kSelWaves];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const uint32_t ntiles = (g.n + (uint32_t)kTile - 1u) / (uint32_t)kTile;
    const uint32_t tile = blockIdx.x * kSelWaves + wave;
    // everything is asked for up front: what there is to know of the tile, the hint record, the window
    TileAhead a0;
    look_ahead(sc, tile, tile < ntiles, a0);
    const uint32_t hint = *sc.hint, hint_shift = sc.hint[kHintShift], hint_hold = sc.hint[kHintHold], hint_cap = sc.hint[kHintCap];
    uint32_t open = wave == kSelWaves - 1 ? sc.hist[kHistOpen + lane] : 0u;      // (the wavefront that holds the window's last bin)
    uint2 wsum = {0u, 0u};                       // window bins 2 t and 2 t + 1
#pragma unroll
    for (int r = 0; r < kWinCopies; ++r) {
        const uint2 x = *reinterpret_cast<const uint2 *>(sc.hist + kHistW + r * kBinsW + 2 * t);
        wsum.x += x.x; wsum.y += x.y;
    }
    // ---- the verdict: the bin b with  count(bins > b) < k <= count(bins >= b), by a suffix scan over the block's
    // threads (two bins each; the counts stay below 2^32, there being fewer elements than that)
    if (wave == kSelWaves - 1) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) open += __shfl_xor(open, d, 64);
        if (lane == 63u) wsum.y += open;         // the last bin also counts every key above the window
    }
    const uint32_t pair = wsum.x + wsum.y;
    const uint32_t pre = wave_scan_incl(pair);
    uint32_t suf = wave_total(pre) - pre + pair;  // inclusive suffix sum: this thread's bins and all above
    if (lane == 0) wtot[wave] = suf;
    if (t == 0) verdict[0] = 0u;
    __syncthreads();
    uint32_t higher = 0, all = 0;                // candidates in the wavefronts after this one; all candidates
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) { if ((uint32_t)w > wave) higher += wtot[w]; all += wtot[w]; }
    suf += higher;
    if ((uint64_t)suf >= k && (uint64_t)(suf - pair) < k) {      // the count crosses k in one of this thread's two bins
        const uint32_t above = suf - pair;
        const bool upper = (uint64_t)above + wsum.y >= k;
        const uint64_t rest = k - above - (upper ? 0u : wsum.y);
        verdict[0] = 1u; verdict[1] = 2u * t + (upper ? 1u : 0u); verdict[2] = (uint32_t)rest; verdict[3] = 0u;
        verdict[6] = upper ? wsum.y : wsum.x;
    }
    if (t == 0) { verdict[4] = all; verdict[5] = 0u; }
    __syncthreads();
    const bool found = verdict[0] != 0u;
    const uint32_t bin = verdict[1];
    const bool first = blockIdx.x == 0 && t == 0;
    if (first) {
        sc.sync[kSyncLastBin] = found ? verdict[6] : 0u;                // diagnostics (mc_select_stats)
        sc.sync[kSyncLastCands] = verdict[4];
    }
    if (found && bin < (uint32_t)kBinsW - 1u) {
        const uint32_t lo = hint + (bin << kWindowShift);
        const bool lean = verdict[6] <= kUCap;
        if (first) {
            SelectState s;
            s.lo = lo; s.mode = kModeFast | (lean ? kModeLean : kModeDense); s.need = (uint64_t)verdict[2] | ((uint64_t)verdict[3] << 32);
            sc.sel[0] = s;
            margin_after_hit(sc.hint, hint_shift, hint_hold, hint_cap, (uint64_t)verdict[4] | ((uint64_t)verdict[5] << 32), k);
            atomicAdd(&sc.sync[kSyncRoutes + (lean ? MC_SELECT_FAST : MC_SELECT_DENSE)], 1u);
        }
        if (!lean) return;               // dense bin: too many keys to list; the slow-route kernel takes its 2048 keys as a radix level
        uint32_t above = 0;
        if (tile < ntiles) {
            const uint32_t sub = tile & (uint32_t)(kUSub - 1);
            MemberBuf mb{members[wave], 0u};
            above = select_tile(sc, a0, lo, sub, mb);
            flush_members(sc, mb, sub);
        }
        // keys above the bin in this block's sixteen tiles
        if (lane == 0) wabove[wave] = above;
        __syncthreads();
        if (t == 0) {
            uint32_t sum = 0;
#pragma unroll
            for (int w = 0; w < kSelWaves; ++w) sum += wabove[w];
            sc.blk_cnt[blockIdx.x] = sum;                          // sixteen tiles hold at most 65536 candidates
        }
        return;
    }
    // missed: the next calls filter with the full margin again, and keep it for a while
    if (first) {
        margin_after_miss(sc.hint, hint_shift, !found);
        SelectState s;
        s.lo = found ? hint + (((uint32_t)kBinsW - 1u) << kWindowShift) : 0u; s.mode = found ? 0u : kModeUniform; s.need = k;
        sc.sel[0] = s;
        atomicAdd(&sc.sync[kSyncRoutes + (found ? MC_SELECT_ABOVE : MC_SELECT_REFILL)], 1u);
    }
}

// The slow routes, in a kernel of their own so that their registers do not weigh on the two kernels of the usual
// route: inside the select kernel they took it to 128 registers and to spilling (one block per compute unit, or two
// tiles per wavefront: 13 .. 30 us instead of 7 .. 10), inside the emit kernel to 108 registers and two rounds of
// blocks.  On the lean route this kernel reads one word and leaves (4 us).
template <int ALGO, bool EF, bool FROM_STATE, bool RANDOM>
__global__ __launch_bounds__(kSelThreads) void sparse_slow_k(GroupView g, float *st, PayloadHeader *hdr, uint64_t k, SparseScratch sc,
                                                             RngKey rng, int *status)
{
    __shared__ __attribute__((aligned(16))) uint32_t hist[kBins1];
    __shared__ uint32_t pfx[2 * kRoundTiles];
    __shared__ uint32_t small[64];
    const SelectState s0 = sc.sel[0];
    if (s0.mode & kModeLean) return;
    slow_routes<ALGO, EF, FROM_STATE, RANDOM>(g, st, hdr, k, sc, rng, s0.mode, s0.lo, s0.need, gridDim.x, status, hist, pfx, small);
}

// Emit, lean route.  One candidate per lane (a chunk's head): gt0 / eq0 count the keys above / equal to T before it
// in the whole group; returns them advanced past these 64.
template <int ALGO, bool EF>
__device__ __forceinline__ void emit_head(uint32_t bits, uint32_t loc, bool valid, uint32_t chunk, uint32_t n, uint64_t k, float *st,
                                          uint32_t *idx, float *val, uint32_t T, uint32_t need, uint64_t &gt0, uint32_t &eq0)
{
    const uint32_t key = bits & 0x7FFFFFFFu;
    const bool is_gt = valid && key > T, is_eq = valid && key == T;
    const uint64_t bgt = __builtin_amdgcn_ballot_w64(is_gt), beq = __builtin_amdgcn_ballot_w64(is_eq);
    const uint64_t gtb = gt0 + lanes_below(bgt);
    const uint32_t eqb = eq0 + lanes_below(beq);
    if (is_gt || (is_eq && eqb < need)) {
        const uint64_t pos = gtb + (eqb < need ? eqb : need);
        const uint32_t i = chunk * (uint32_t)kChunk + loc;
        if (pos < k && i < n) {                  // always true for consistent scratch
            idx[pos] = i;
            if (ALGO == MC_ALGO_RANDK) val[pos] = st[i];      // the candidate slot holds the random key: the value is p
            else val[pos] = __uint_as_float(bits);
            drop_sent<ALGO, EF>(st, n, i, is_eq);
        }
    }
    gt0 += __popcll(bgt); eq0 += __popcll(beq);
}

// ... four consecutive candidates per lane (a unit; it holds at most 256 keys above T and as many equal to it)
template <int ALGO, bool EF>
__device__ __forceinline__ void emit_unit(const uint4 &bits, const uint2 &loc, uint32_t cnt, uint32_t v, uint32_t chunk, uint32_t n,
                                          uint64_t k, float *st, uint32_t *idx, float *val, uint32_t T, uint32_t need, uint64_t &gt0, uint32_t &eq0)
{
    bool isg[4], ise[4];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t key = elem4(bits, j) & 0x7FFFFFFFu;
        const bool valid = in_unit(cnt, v, j);
        isg[j] = valid && key > T; ise[j] = valid && key == T;
        mine += (isg[j] ? 1u : 0u) + (ise[j] ? 0x10000u : 0u);
    }
    const uint32_t inc = wave_scan_incl(mine);
    const uint32_t tot = wave_total(inc);
    uint64_t gtb = gt0 + ((inc - mine) & 0xFFFFu);
    uint32_t eqb = eq0 + ((inc - mine) >> 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (isg[j] || (ise[j] && eqb < need)) {
            const uint64_t pos = gtb + (eqb < need ? eqb : need);
            const uint32_t i = chunk * (uint32_t)kChunk + loc4(loc, j);
            if (pos < k && i < n) {
                idx[pos] = i;
                if (ALGO == MC_ALGO_RANDK) val[pos] = st[i];
                else val[pos] = __uint_as_float(elem4(bits, j));
                drop_sent<ALGO, EF>(st, n, i, ise[j]);
            }
        }
        gtb += isg[j] ? 1u : 0u; eqb += ise[j] ? 1u : 0u;
    }
    gt0 += tot & 0xFFFFu; eq0 += tot >> 16;
}

// Emit: four tiles per block, one wavefront each.  Every block reads the whole list of the keys in the threshold's
// bin (it is small), finds the threshold key T and the number of keys equal to T to take with a histogram in LDS,
// counts the list's kept keys that lie before each of its tiles, adds the keys above the bin in the tiles before,
// and compacts its tiles' kept candidates into the payload.  The heads of the tile's chunks and the first entries
// of every sublist are asked for together with everything else, so the usual tile costs one memory latency.
// Consecutive entries that a thread of an emit block fetches before the sublists' lengths are known, four threads per
// sublist: a list of a few hundred keys (9 per sublist) is then complete after the first level of loads.  Measured
// with 1 / 2 / 4 / 8: emit 13.6 / 13.5 / 13.0 / 13.8 us on the bench's Top-k, whole compress 82.7 / 82.1 / 80.1 / 78.0
// where the bin holds 2500 keys (tensors of one scale), DGC and Rand-k +1 us with 8 (68 registers instead of 60).
constexpr int kUPer = 4;
constexpr int kUSpec = 4 * kUPer;      // ... which covers the first kUSpec entries of every sublist
static_assert(4 * kUSub == kEmitThreads, "four threads per sublist");

template <int ALGO, bool EF>
__global__ __launch_bounds__(kEmitThreads) void lean_emit_k(uint32_t n, uint32_t ntiles, float *st, PayloadHeader *hdr, uint64_t k,
                                                            SparseScratch sc)
{
    __shared__ uint32_t hist[kBins3], coarse[64];          // the listed keys' 11 open bits, and the same 32 bins at a time
    __shared__ uint32_t small[4];
    __shared__ uint32_t ulen[kUSub], upre[kUSub + 1];
    __shared__ uint32_t cgt[kEmitWaves + 1], ceq[kEmitWaves + 1];
    __shared__ uint32_t red[kEmitWaves];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const uint32_t tile = blockIdx.x * kEmitWaves + wave;
    const bool live = tile < ntiles;
    // ---- everything that needs no other load to be located is asked for now
    const uint64_t runs = live ? sc.tile_runs[tile] : 0ull;
    const SelectState s0 = sc.sel[0];
    const uint32_t ucnt = wave == 0 ? sc.ucount[lane * kUCountStride] : 0u;
    UEntry spec[kUPer];                                    // entries (t % 4) kUPer ... of sublist t / 4, if it has that many
#pragma unroll
    for (int i = 0; i < kUPer; ++i) spec[i] = sc.ulist[(size_t)(t / 4u) * kUCap + (t % 4u) * kUPer + i];
    uint32_t hb[kWavesPerBlock], hl[kWavesPerBlock];
#pragma unroll
    for (int q = 0; q < kWavesPerBlock; ++q) {
        hb[q] = live ? load_head_bits(sc, tile * kWavesPerBlock + q) : 0u;
        hl[q] = live ? load_head_loc(sc, tile * kWavesPerBlock + q) : 0u;
    }
    // ... and, as soon as the counts are there, the first four units of a tile with crowded chunks (nearly always all it has)
    uint32_t cnt[kWavesPerBlock];
#pragma unroll
    for (int q = 0; q < kWavesPerBlock; ++q) cnt[q] = (uint32_t)(runs >> (16 * q)) & 0xFFFFu;
    const TileUnits tu(cnt);
    uint4 kb[4];
    uint2 kl[4];
    uint32_t kq[4], kv[4];
    if (tu.total) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            tu.locate((uint32_t)i < tu.total ? (uint32_t)i : 0u, kq[i], kv[i]);
            kb[i] = load_bits4(sc, tile * kWavesPerBlock + kq[i], kv[i]);
            kl[i] = load_loc4(sc, tile * kWavesPerBlock + kq[i], kv[i]);
        }
    }
    // keys above the bin in the select blocks (sixteen tiles each) before this tile's, then in the tiles before it in its own
    const uint32_t sblock = tile / (uint32_t)kSelWaves, sfirst = sblock * (uint32_t)kSelWaves;
    uint32_t before = 0;
    for (uint32_t b = t; b < blockIdx.x / (uint32_t)(kSelWaves / kEmitWaves); b += kEmitThreads) before += sc.blk_cnt[b];
    uint32_t mine = live && sfirst + lane < tile ? sc.tile_cnt[sfirst + lane] : 0u;
    // the select kernel is done with the window: all blocks clear it together
    for (uint32_t b = blockIdx.x * kEmitThreads + t; b < (uint32_t)(kWinCopies * kBinsW + kOpenCopies); b += gridDim.x * kEmitThreads)
        sc.hist[b < (uint32_t)(kWinCopies * kBinsW) ? kHistW + b : kHistOpen - kWinCopies * kBinsW + b] = 0u;
    if (!(s0.mode & kModeLean)) return;                 // (the slow routes have written the payload themselves)
    const uint32_t lo = s0.lo;
    // ---- the list
    if (wave == 0) {
        const uint32_t len = min(ucnt, kUCap);
        ulen[lane] = len;
        const uint32_t inc = wave_scan_incl(len > (uint32_t)kUSpec ? len - (uint32_t)kUSpec : 0u);      // entries beyond the speculative ones, scanned
        upre[lane + 1] = inc;
        if (lane == 0) upre[0] = 0u;
    }
    for (int b = t; b < kBins3; b += kEmitThreads) hist[b] = 0u;
    if (t < 64u) coarse[t] = 0u;
    if (t <= (uint32_t)kEmitWaves) { cgt[t] = 0u; ceq[t] = 0u; }
    __syncthreads();
    const uint32_t spec_n = ulen[t / 4u] > (t % 4u) * kUPer ? min(ulen[t / 4u] - (t % 4u) * kUPer, (uint32_t)kUPer) : 0u;      // of spec[], this many exist
    const uint32_t more = min(upre[kUSub], kUCap);       // (nothing, when no sublist holds more than four entries)
    // further entry e: entry kUSpec + (e - upre[s]) of the sublist s that is the last to start at or before e
    auto further = [&](uint32_t e) {
        uint32_t sl = 0;
#pragma unroll
        for (int step = kUSub / 2; step >= 1; step >>= 1) if (upre[sl + step] <= e) sl += step;
        return sc.ulist[(size_t)sl * kUCap + kUSpec + (e - upre[sl])];
    };
    auto tally = [&](uint32_t bits) {
        const uint32_t d = (bits & 0x7FFFFFFFu) - lo;
        if (d < (uint32_t)kBins3) { atomicAdd(&hist[d], 1u); atomicAdd(&coarse[d >> 5], 1u); }
    };
#pragma unroll
    for (int i = 0; i < kUPer; ++i) if ((uint32_t)i < spec_n) tally(spec[i].bits);
    for (uint32_t e0 = t; e0 < more; e0 += 4 * kEmitThreads) {        // (four loads in flight)
        UEntry x[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) if (e0 + i * kEmitThreads < more) x[i] = further(e0 + i * kEmitThreads);
#pragma unroll
        for (int i = 0; i < 4; ++i) if (e0 + i * kEmitThreads < more) tally(x[i].bits);
    }
    __syncthreads();
    // threshold key and the number of keys equal to it to take: the key at which the count from the top reaches
    // s0.need, first among the 64 coarse bins, then among the 32 keys of that one
    if (wave == 0) {
        const uint32_t want = (uint32_t)s0.need;           // (at most kUCap)
        const uint32_t c = coarse[lane];
        const uint32_t cpre = wave_scan_incl(c);
        const uint32_t suf = wave_total(cpre) - cpre + c;          // from the top
        const uint64_t hit = __builtin_amdgcn_ballot_w64(suf >= want && suf - c < want);
        uint32_t b = 0, r = 0;
        if (hit) {
            const uint32_t cl = (uint32_t)__builtin_ctzll(hit);
            const uint32_t left = want - (__shfl(suf, cl, 64) - __shfl(c, cl, 64));      // to take inside the coarse bin
            const uint32_t f = lane < 32u ? hist[32u * cl + lane] : 0u;
            const uint32_t fpre = wave_scan_incl(f);
            const uint32_t fs = wave_total(fpre) - fpre + f;
            const uint64_t hit2 = __builtin_amdgcn_ballot_w64(lane < 32u && fs >= left && fs - f < left);
            if (hit2) {
                const uint32_t fl = (uint32_t)__builtin_ctzll(hit2);
                b = 32u * cl + fl;
                r = left - (__shfl(fs, fl, 64) - __shfl(f, fl, 64));
            }
        }
        if (lane == 0) { small[0] = b; small[1] = r; }       // (an inconsistent list: T = lo, nothing equal taken)
    }
    __syncthreads();
    const uint32_t T = lo + small[0], need = small[1];
    // the list's kept keys, by where they lie: before this block, or in its tile j (bucket j + 1)
    const uint32_t first = blockIdx.x * (uint32_t)(kEmitWaves * kTile);
    auto classify = [&](const UEntry &x) {
        const uint32_t key = x.bits & 0x7FFFFFFFu;
        if (key >= T) {
            const uint32_t bucket = x.idx < first ? 0u : ((x.idx - first) >> 12) + 1u;
            if (bucket <= (uint32_t)kEmitWaves) atomicAdd(key > T ? &cgt[bucket] : &ceq[bucket], 1u);
        }
    };
#pragma unroll
    for (int i = 0; i < kUPer; ++i) if ((uint32_t)i < spec_n) classify(spec[i]);
    for (uint32_t e0 = t; e0 < more; e0 += 4 * kEmitThreads) {
        UEntry x[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) if (e0 + i * kEmitThreads < more) x[i] = further(e0 + i * kEmitThreads);
#pragma unroll
        for (int i = 0; i < 4; ++i) if (e0 + i * kEmitThreads < more) classify(x[i]);
    }
    before = wave_total(wave_scan_incl(before));          // (sums of candidates: below 2^32)
    mine = wave_total(wave_scan_incl(mine));
    if (lane == 0) red[wave] = before;
    __syncthreads();
    if (blockIdx.x == 0 && t == 0) { put_sparse_header(hdr, ALGO, n, k); publish_hint(sc, T); record_sent_key<ALGO, EF>(st, T); }
    if (!live) return;
    uint64_t gt0 = mine;
    uint32_t eq0;
#pragma unroll
    for (int w = 0; w < kEmitWaves; ++w) gt0 += red[w];
    {
        uint32_t g2 = 0, e2 = 0;                            // the list's kept keys before this tile: buckets 0 .. wave
#pragma unroll
        for (int b = 0; b <= kEmitWaves; ++b) if ((uint32_t)b <= wave) { g2 += cgt[b]; e2 += ceq[b]; }
        gt0 += g2; eq0 = e2;
    }
    uint32_t *idx = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(hdr) + kHeaderBytes);
    float *val = reinterpret_cast<float *>(idx + k);
    if (lane == 0) {
        uint32_t *dir = payload_directory(hdr, k);
        dir[tile] = (uint32_t)(gt0 + (eq0 < need ? eq0 : need));
        if (tile == ntiles - 1u) dir[ntiles] = (uint32_t)k;              // (the selection keeps exactly k)
    }
    if (tu.total == 0) {
        // the usual tile: no chunk holds more than 64 candidates, and they are all here
#pragma unroll
        for (int q = 0; q < kWavesPerBlock; ++q)
            if (cnt[q]) emit_head<ALGO, EF>(hb[q], hl[q], lane < cnt[q], tile * kWavesPerBlock + q, n, k, st, idx, val, T, need, gt0, eq0);
        return;
    }
    // A tile with crowded chunks: its pieces -- the head of chunk 0, its units, the head of chunk 1, ... -- are placed in
    // index order, the counts of kept keys running along.  Up to four units, nearly every such tile, were fetched at
    // the start; a tile with more fetches them four at a time.  One copy of the unit's code in a loop that is not
    // unrolled: sixteen unrolled copies were 2 us slower (code size), and counting all pieces first, scanning the counts
    // and fetching the units of a very crowded tile a second time 1.3 us slower (Top-k emit 13.0 -> 11.7 us).
    uint32_t e = 0;                                         // next unit of the tile
#pragma unroll
    for (int q = 0; q < kWavesPerBlock; ++q) {
        const uint32_t cq = cnt[q];
        if (!cq) continue;
        emit_head<ALGO, EF>(hb[q], hl[q], lane < cq, tile * kWavesPerBlock + q, n, k, st, idx, val, T, need, gt0, eq0);
        const uint32_t nu = tu.per[q];
#pragma unroll 1
        for (uint32_t v = 0; v < nu; ++v, ++e) {
            if (e >= 4u && (e & 3u) == 0u) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    tu.locate(e + i < tu.total ? e + i : e, kq[i], kv[i]);
                    kb[i] = load_bits4(sc, tile * kWavesPerBlock + kq[i], kv[i]);
                    kl[i] = load_loc4(sc, tile * kWavesPerBlock + kq[i], kv[i]);
                }
            }
            // unit e % 4 of the four in registers, chosen word by word (an array indexed at run time would live in scratch memory)
            const uint32_t s = e & 3u;
            auto sel = [s](uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3) { return s == 0u ? a0 : s == 1u ? a1 : s == 2u ? a2 : a3; };
            uint4 b;
            b.x = sel(kb[0].x, kb[1].x, kb[2].x, kb[3].x); b.y = sel(kb[0].y, kb[1].y, kb[2].y, kb[3].y);
            b.z = sel(kb[0].z, kb[1].z, kb[2].z, kb[3].z); b.w = sel(kb[0].w, kb[1].w, kb[2].w, kb[3].w);
            uint2 l;
            l.x = sel(kl[0].x, kl[1].x, kl[2].x, kl[3].x); l.y = sel(kl[0].y, kl[1].y, kl[2].y, kl[3].y);
            emit_unit<ALGO, EF>(b, l, cq, v, tile * kWavesPerBlock + q, n, k, st, idx, val, T, need, gt0, eq0);
        }
    }
}

template <int ALGO, bool EF, bool CAPPED>
static void sparse_compress_t(const LaunchCtx &lc, const GroupView &g, float *st, float momentum, uint64_t k, uint64_t need,
                              PayloadHeader *hdr, const SparseScratch &sc, const RngKey &rng, const SampleRule &smp,
                              uint32_t sync_blocks, int *status)
{
    constexpr bool FS = (ALGO == MC_ALGO_DGC) || EF;
    constexpr bool RND = ALGO == MC_ALGO_RANDK;
    const uint32_t nt = tiles_of(g.n), nch = chunks_of(g.n);
    const uint32_t sblocks = (nch + 15) / 16 < 256 ? (nch + 15) / 16 : 256;      // enough to stream the group in a refill
    dim3 grid(nt), block(kBlock), cgrid((nt + kWavesPerBlock - 1) / kWavesPerBlock);
    prof_begin(lc, K_SPARSE_ACCUM);
    MC_LAUNCH((sparse_accum_k<ALGO, EF>), grid, block, lc, g, st, momentum, sc, rng, smp);
    prof_end(lc, K_SPARSE_ACCUM);
    if (!CAPPED) {
        // the two-kernel tail; its slow routes run on at most `sync_blocks` blocks, which the device holds at once
        const uint32_t sblocks = (nt + kSelWaves - 1) / kSelWaves, eblocks = (nt + kEmitWaves - 1) / kEmitWaves;
        // the slow routes run on blocks that the device holds at once: one per compute unit
        const uint32_t sync = std::max(1u, std::min(std::min(sync_blocks, sblocks), (uint32_t)(kRoundTiles / kSelWaves)));
        prof_begin(lc, K_LEAN_SELECT);
        MC_LAUNCH(lean_select_k, dim3(sblocks), dim3(kSelThreads), lc, g, k, sc);
        prof_end(lc, K_LEAN_SELECT);
        prof_begin(lc, K_SPARSE_SLOW);
        MC_LAUNCH((sparse_slow_k<ALGO, EF, FS, RND>), dim3(sync), dim3(kSelThreads), lc, g, st, hdr, k, sc, rng, status);
        prof_end(lc, K_SPARSE_SLOW);
        prof_begin(lc, K_LEAN_EMIT);
        MC_LAUNCH((lean_emit_k<ALGO, EF>), dim3(eblocks), dim3(kEmitThreads), lc, g.n, nt, st, hdr, k, sc);
        prof_end(lc, K_LEAN_EMIT);
        return;
    }
    prof_begin(lc, K_SPARSE_SEED);
    MC_LAUNCH((sparse_seed_k<FS, RND>), dim3(sblocks), dim3(kSeedThreads), lc, g, st, need, sc, rng, smp);
    prof_end(lc, K_SPARSE_SEED);
    prof_begin(lc, K_CAND_HIST2);
    MC_LAUNCH(cand_hist_k<2>, cgrid, block, lc, g.n, nt, sc, smp);
    prof_end(lc, K_CAND_HIST2);
    prof_begin(lc, K_CAND_HIST3);
    MC_LAUNCH(cand_hist_k<3>, cgrid, block, lc, g.n, nt, sc, smp);
    prof_end(lc, K_CAND_HIST3);
    prof_begin(lc, K_CAND_COUNT);
    MC_LAUNCH(cand_count_k, cgrid, block, lc, g.n, nt, sc);
    prof_end(lc, K_CAND_COUNT);
    prof_begin(lc, K_CAND_EMIT);
    MC_LAUNCH((cand_emit_k<ALGO, EF, CAPPED>), cgrid, block, lc, g.n, nt, st, hdr, k, sc);
    prof_end(lc, K_CAND_EMIT);
}

// k: entries of the payload (the exact k, or the capacity when the threshold comes from a sample);
// sample_stride > 0: DGC with a sampled threshold, the sample starts at sample_first and the threshold is its
// sample_need-th largest key
void launch_sparse_compress(const LaunchCtx &lc, int algo, const GroupView &g, bool ef, float *state_f, float momentum,
                            uint64_t k, PayloadHeader *hdr, const SparseScratch &sc, uint64_t seed, uint32_t worker, uint32_t iter_lo,
                            uint32_t sample_stride, uint32_t sample_first, uint64_t sample_need, uint32_t sync_blocks, int *status)
{
    if (g.n == 0) return;
    const RngKey rng{seed, worker, iter_lo};
    SampleRule smp{0u, 0u, 0u};
    if (algo == MC_ALGO_DGC && sample_stride) {
        smp.stride = sample_stride; smp.first = sample_first;
        smp.inv = sample_stride > 1 ? (uint32_t)((1ull << 32) / sample_stride) : 0u;
        sparse_compress_t<MC_ALGO_DGC, true, true>(lc, g, state_f, momentum, k, sample_need, hdr, sc, rng, smp, sync_blocks, status);
    } else if (algo == MC_ALGO_DGC) sparse_compress_t<MC_ALGO_DGC, true, false>(lc, g, state_f, momentum, k, k, hdr, sc, rng, smp, sync_blocks, status);
    else if (algo == MC_ALGO_RANDK) sparse_compress_t<MC_ALGO_RANDK, true, false>(lc, g, state_f, momentum, k, k, hdr, sc, rng, smp, sync_blocks, status);
    else if (ef) sparse_compress_t<MC_ALGO_TOPK, true, false>(lc, g, state_f, momentum, k, k, hdr, sc, rng, smp, sync_blocks, status);
    else sparse_compress_t<MC_ALGO_TOPK, false, false>(lc, g, state_f, momentum, k, k, hdr, sc, rng, smp, sync_blocks, status);
}

// ---------------------------------------------------------------------------
// Sparse decompress-and-sum.  Every worker's indices ascend, so a 4096-element
// output tile owns one contiguous run of each list, and the directory that ends a
// payload says where that run starts and ends.  A block accumulates its tile in LDS,
// one worker after the other in ascending worker order -- the same order of fp32
// additions as a dense sum, since adding the +0 of an absent entry changes nothing --
// and writes it once.  No atomics, no pre-zeroed output, bit-reproducible.
// (The directory replaced a kernel that recorded the runs of all payloads in per-call
// tables before this one could start: 5 of 38 us.)
// ---------------------------------------------------------------------------
constexpr int kSparseBatch = 8;    // workers whose entries are in flight together
// rounds of 256 entries per worker fetched up front (with 4 the kernel needs 74 vector registers and 6 wavefronts
// fit a SIMD; with 3, 58 and 8: measured 0.7 .. 1.9 us faster, 2 rounds no better)
constexpr int kSparseRounds = 3;

// k64: entries a payload has room for (the exact k, or the capacity when DGC takes its threshold from a sample: the
// header then says how many are in use and repeats the capacity)
__global__ __launch_bounds__(kBlock) void sparse_decompress_k(int algo, GroupView out, PayloadPtrs pl, int W, float alpha,
                                                              uint64_t k64, uint32_t ntiles, int *status, int capped)
{
    __shared__ float acc[kTile];
    const uint32_t k = (uint32_t)k64;
    if (blockIdx.x == 0 && (int)threadIdx.x < W) {
        const PayloadHeader *h = reinterpret_cast<const PayloadHeader *>(pl.p[threadIdx.x]);
        const bool fits = capped ? h->k <= k64 && h->levels == (uint32_t)k64 : h->k == k64;
        if (h->magic != kMagic || h->algo != (uint32_t)algo || h->n != (uint64_t)out.n || !fits) *status = 1;
    }
    const uint32_t tile = my_tile_index();
    const uint32_t tb = tile * (uint32_t)kTile;
    const uint32_t t = threadIdx.x;
    const Chunk c = my_chunk(out.n, tile);
    const uintptr_t entry = chunk_entry(out, c);        // needed last, asked for first: overlaps with the table loads
    if (W > kSparseBatch) {
        // more workers than one batch: the tiles that no worker has an entry for are found first, over all batches
        // (the per-batch test below only sees its own eight), and zero-filled as with one batch
        bool any = false;
        for (int w = 0; w < W; ++w) {
            const uint32_t *dir = reinterpret_cast<const uint32_t *>(pl.p[w] + kHeaderBytes + 8u * k64);
            const uint32_t f = ld_uniform(dir + tile), l = ld_uniform(dir + tile + 1u);
            any = any || (l < k ? l : k) > (f < k ? f : k);
        }
        if (!any) {
            if (c.base >= out.n) return;
            float z[kSteps];
#pragma unroll
            for (int j = 0; j < kSteps; ++j) z[j] = alpha * 0.0f;
            store_seg_rot(out, c, z, entry, chunk_rotation(entry));
            return;
        }
    }
    for (int w0 = 0; w0 < W; w0 += kSparseBatch) {
        // issue the loads of a batch of workers before the first LDS update
        uint32_t lo[kSparseBatch], hi[kSparseBatch];
#pragma unroll
        for (int b = 0; b < kSparseBatch; ++b) {
            lo[b] = hi[b] = 0;
            if (w0 + b < W) {
                // block-uniform addresses, kept on the scalar path whatever the compiler makes of the rest
                const uint32_t *dir = reinterpret_cast<const uint32_t *>(pl.p[w0 + b] + kHeaderBytes + 8u * k64);
                const uint32_t f = ld_uniform(dir + tile), l = ld_uniform(dir + tile + 1u);
                lo[b] = f < k ? f : k;
                hi[b] = l < k ? l : k;
                // inconsistent payload (a directory that does not ascend): a tile holds at most 4096 entries
                if (hi[b] < lo[b] || hi[b] - lo[b] > (uint32_t)kTile) hi[b] = lo[b];
            }
        }
        if (W <= kSparseBatch) {          // most tiles hold no kept entry at all: they are just zero-filled
            bool any = false;
#pragma unroll
            for (int b = 0; b < kSparseBatch; ++b) any = any || hi[b] > lo[b];
            if (!any) {
                if (c.base >= out.n) return;
                float z[kSteps];
#pragma unroll
                for (int j = 0; j < kSteps; ++j) z[j] = alpha * 0.0f;
                // whole lines per wave store (measured: -0.5 us; the same rotation on the path below costs 3 us)
                store_seg_rot(out, c, z, entry, chunk_rotation(entry));
                return;
            }
        }
        if (W <= kSparseBatch) {
            // Few entries per worker (at most one per lane): every wavefront sums its own chunk, in LDS of its own, from
            // the tile's entries of all workers -- loaded together, added worker by worker, no block barrier.  The LDS
            // operations of one wavefront complete in the order issued, so a worker's additions see the ones before.
            bool light = true;
#pragma unroll
            for (int b = 0; b < kSparseBatch; ++b) light = light && hi[b] - lo[b] <= 64u;
            if (light) {
                if (c.base >= out.n) return;
                uint32_t ix[kSparseBatch];
                float vv[kSparseBatch];
#pragma unroll
                for (int b = 0; b < kSparseBatch; ++b) {
                    const uint32_t *idx = reinterpret_cast<const uint32_t *>(pl.p[b < W ? b : 0] + kHeaderBytes);
                    const float *val = reinterpret_cast<const float *>(idx + k);
                    const uint32_t e = lo[b] + c.lane;
                    ix[b] = 0xFFFFFFFFu; vv[b] = 0.0f;
                    if (b < W && e < hi[b]) { ix[b] = ld_stream(idx + e); vv[b] = ld_stream(val + e); }
                }
                float *mine = acc + (c.base - tb);
#pragma unroll
                for (int j = 0; j < kSteps; ++j) mine[64 * j + c.lane] = 0.0f;
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int b = 0; b < kSparseBatch; ++b) {
                    const uint32_t local = ix[b] - c.base;          // an absent entry (all ones) lands far outside
                    if (b < W && local < (uint32_t)kChunk) mine[local] = mine[local] + vv[b];
                    __builtin_amdgcn_wave_barrier();
                }
                // read back in the mapping rotated onto the output's 128-byte lines (payloads spread thinly over all
                // tiles: 37.2 -> 36.3 us; clustered ones: 32.3 -> 32.1; the same on the path below changes nothing)
                float v[kSteps];
                const uint32_t rot = chunk_rotation(entry);
#pragma unroll
                for (int j = 0; j < kSteps; ++j) v[j] = alpha * mine[rotated(j, c.lane, rot)];
                store_seg_rot(out, c, v, entry, rot);
                return;
            }
        }
        if (w0 == 0) {
#pragma unroll
            for (int j = 0; j < kSteps; ++j) acc[t + kBlock * j] = 0.0f;
            __syncthreads();
        }
        // the kept entries cluster in a few tensors: a tile there holds hundreds of entries per worker.
        // Three rounds of 256 entries of every worker of the batch are requested at once.
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
    if (c.base >= out.n) return;
    float v[kSteps];
    const float *mine = acc + (c.base - tb) + c.lane;
#pragma unroll
    for (int j = 0; j < kSteps; ++j) v[j] = alpha * mine[64 * j];
    store_seg(out, c, v, entry);
}

void launch_sparse_decompress(const LaunchCtx &lc, int algo, const GroupView &out, const PayloadPtrs &pl, int W,
                              float alpha, uint64_t k, int *status, bool capped)
{
    if (out.n == 0) return;
    const uint32_t nt = tiles_of(out.n);
    prof_begin(lc, K_SPARSE_DECOMPRESS);
    MC_LAUNCH(sparse_decompress_k, dim3(nt), dim3(kBlock), lc, algo, out, pl, W, alpha, k, nt, status, capped ? 1 : 0);
    prof_end(lc, K_SPARSE_DECOMPRESS);
}

}  // namespace mc
