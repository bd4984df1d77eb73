// Dense-code compressors (EF-Sign, QSGD, TernGrad, FP16) and their
// decompress-and-sum, for gfx950.  One launch covers a whole merged group
// (Section 4.1 of the paper: the tensors of a group are compressed in one
// operation); tensors are reached through the segment table, nothing is copied.
//
// All kernels are HBM-streaming: each operand is touched once per pass with
// lane-consecutive 4-byte accesses (256 contiguous bytes per wave instruction),
// sign / ternary planes are packed with 64-lane ballots, group scalars are
// reduced per block in LDS and combined by a one-block finalize kernel.
#include <cstddef>

#include "mc_internal.h"

namespace mc {

// ---------------------------------------------------------------------------
// pointer-table upload: the per-call list of tensor addresses travels in the
// kernel argument buffer, so no host staging memory has to outlive the call.
// ---------------------------------------------------------------------------
__global__ void upload_ptrs_k(PtrChunk chunk, uintptr_t *dst, uint32_t count)
{
    uint32_t i = threadIdx.x;
    if (i < count) dst[i] = chunk.p[i];
}

void launch_upload_ptrs(const LaunchCtx &lc, const uintptr_t *host, uintptr_t *dev, uint32_t count)
{
    for (uint32_t done = 0; done < count; done += 256) {
        PtrChunk ch;
        uint32_t m = count - done < 256 ? count - done : 256;
        for (uint32_t i = 0; i < 256; ++i) ch.p[i] = i < m ? host[done + i] : 0;
        prof_begin(lc, K_UPLOAD);
        MC_LAUNCH(upload_ptrs_k, dim3(1), dim3(256), lc, ch, dev + done, m);
        prof_end(lc, K_UPLOAD);
    }
}

// Per-chunk address table of a freshly uploaded tensor address list: the address of
// the chunk's first element when all 1024 elements lie in one tensor, else 2 s + 1 with s the tensor of its first element.
__global__ __launch_bounds__(kBlock) void expand_ptrs_k(GroupView g, uintptr_t *chunk_addr)
{
    const uint32_t nchunks = (g.n + (uint32_t)kChunk - 1u) / (uint32_t)kChunk;
    const uint32_t c = blockIdx.x * kBlock + threadIdx.x;
    if (c >= nchunks) return;
    const uint32_t base = c * (uint32_t)kChunk;
    const uint32_t s = g.chunk_seg[c];
    const uint32_t beg = g.seg_off[s], end = g.seg_off[s + 1];
    uintptr_t a = ((uintptr_t)s << 1) | 1u;            // not an address: where the loop over the chunk's tensors starts
    if (g.n - base >= (uint32_t)kChunk && end - base >= (uint32_t)kChunk) a = g.ptrs[s] + (uintptr_t)(base - beg) * sizeof(float);
    chunk_addr[c] = a;
}

void launch_expand_ptrs(const LaunchCtx &lc, const GroupView &g, uintptr_t *chunk_addr)
{
    if (g.n == 0) return;
    const uint32_t nchunks = (uint32_t)(((uint64_t)g.n + kChunk - 1) / kChunk);
    prof_begin(lc, K_UPLOAD);
    MC_LAUNCH(expand_ptrs_k, dim3((nchunks + kBlock - 1) / kBlock), dim3(kBlock), lc, g, chunk_addr);
    prof_end(lc, K_UPLOAD);
}

static inline uint32_t tiles_of(uint32_t n) { return (uint32_t)(((uint64_t)n + kTile - 1) / kTile); }

// ---------------------------------------------------------------------------
// The one-bit schemes, single pass: one sign bit per element of a vector p.
//   SIGN_EF       EF-Sign: delta = (||p||_1 / n) sign(p), p = g + e, e <- p - delta
//   SIGN_MEANS    OneBit: delta = mean of the class (p >= 0 / p < 0) of the element, same residual rule
//   SIGN_PLAIN    SignSGD: p = g, nothing is remembered
//   SIGN_MOMENTUM SigNUM: p = m <- beta m + (1 - beta) g, the momentum is the state
// The bits of the first two do not depend on their group scalars, so the residual is
// not written: the state keeps p and the scalars of the call that produced it, and
// the residual of the previous call is re-derived on the fly as
//     e = p_prev - (p_prev >= 0 ? hi_prev : lo_prev)          (EF-Sign: hi = s, lo = -s)
// with the same fp32 operations an explicit update would have used.
// Traffic per element: read g, read p_prev, write p, 1/8 byte of sign bits.
// Per-block partials: EF-Sign sum |p|; OneBit sum of the upper class, sum of the lower
// class, size of the upper class (three arrays of gridDim.x doubles).
// ---------------------------------------------------------------------------
// header of a payload whose group scalar needs no reduction (written by one thread of the compress kernel itself)
__device__ __forceinline__ void put_plain_header(PayloadHeader *hdr, uint32_t algo, uint32_t n, float scale)
{
    PayloadHeader h;
    h.magic = kMagic; h.algo = algo; h.n = n; h.k = 0; h.scale = scale; h.levels = 0;
    for (int i = 0; i < 24; ++i) h.pad[i] = 0;
    *hdr = h;
}

template <int MODE, bool EF>
__global__ __launch_bounds__(kBlock) void sign_compress_k(GroupView g, float *st, const StateHeader *prev, float beta,
                                                          uint32_t *words, uint32_t nwords, double *partial,
                                                          PayloadHeader *hdr, uint32_t algo)
{
    __shared__ uint64_t stage[kWavesPerBlock][kSteps];
    __shared__ double red[kWavesPerBlock];
    __shared__ double red3[MODE == SIGN_MEANS ? 3 : 1][kWavesPerBlock];
    const Chunk c = my_chunk(g.n);
    // SignSGD, SigNUM: the decoded values are +-1, no finalize kernel follows
    if ((MODE == SIGN_PLAIN || MODE == SIGN_MOMENTUM) && blockIdx.x == 0 && threadIdx.x == 0) put_plain_header(hdr, algo, g.n, 1.0f);
    double acc = 0.0, acc_lo = 0.0, cnt_hi = 0.0;
    if (c.base < g.n) {
        float p[kSteps];
        load_seg(g, c, p);
        if (MODE == SIGN_MOMENTUM) {
            const float omb = 1.0f - beta;
            float q[kSteps];
            load_flat(st, c, g.n, q, 0.0f);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                const float bm = beta * q[j], og = omb * p[j];
                p[j] = bm + og;
            }
            store_flat(st, c, g.n, p);
        } else if (EF && MODE != SIGN_PLAIN) {
            const float hi = prev->scale, lo = MODE == SIGN_MEANS ? prev->scale_lo : -hi;
            float q[kSteps];
            load_flat(st, c, g.n, q, 0.0f);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                float d = q[j] >= 0.0f ? hi : lo;
                float e = q[j] - d;
                p[j] = p[j] + e;
            }
            store_flat(st, c, g.n, p);
        }
        uint64_t b[kSteps];
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            bool valid = c.full || (c.base + 64 * j + c.lane < g.n);
            const bool up = valid && p[j] >= 0.0f;
            b[j] = __builtin_amdgcn_ballot_w64(up);
            if (MODE == SIGN_EF) acc += valid ? fabs((double)p[j]) : 0.0;
            if (MODE == SIGN_MEANS) {
                acc += up ? (double)p[j] : 0.0;
                acc_lo += valid && !up ? (double)p[j] : 0.0;
            }
        }
        if (MODE == SIGN_MEANS) {
#pragma unroll
            for (int j = 0; j < kSteps; ++j) if (c.lane == 0) cnt_hi += (double)__popcll(b[j]);
        }
        store_plane(words, nwords, c, b, stage[threadIdx.x >> 6]);
    }
    if (MODE == SIGN_EF) {
        double t = block_sum(acc, red);
        if (threadIdx.x == 0) partial[my_tile_index()] = t;
    }
    if (MODE == SIGN_MEANS) {       // the three sums behind one pair of barriers, each combined in block_sum's order
        acc = wave_sum(acc); acc_lo = wave_sum(acc_lo); cnt_hi = wave_sum(cnt_hi);
        if ((threadIdx.x & 63) == 0) { red3[0][threadIdx.x >> 6] = acc; red3[1][threadIdx.x >> 6] = acc_lo; red3[2][threadIdx.x >> 6] = cnt_hi; }
        __syncthreads();
        if (threadIdx.x < 3)
            partial[threadIdx.x * gridDim.x + my_tile_index()] = (red3[threadIdx.x][0] + red3[threadIdx.x][1]) + (red3[threadIdx.x][2] + red3[threadIdx.x][3]);
    }
}

void launch_sign_compress(const LaunchCtx &lc, int mode, const GroupView &g, bool ef, float *state_f, const StateHeader *prev,
                          float beta, uint32_t *words, uint32_t nwords, double *partial, PayloadHeader *hdr, uint32_t algo)
{
    if (g.n == 0) return;
    dim3 grid(tiles_of(g.n)), block(kBlock);
    prof_begin(lc, K_EFSIGN_COMPRESS);
    switch (mode) {
    case SIGN_EF:
        if (ef) MC_LAUNCH((sign_compress_k<SIGN_EF, true>), grid, block, lc, g, state_f, prev, beta, words, nwords, partial, hdr, algo);
        else MC_LAUNCH((sign_compress_k<SIGN_EF, false>), grid, block, lc, g, state_f, prev, beta, words, nwords, partial, hdr, algo);
        break;
    case SIGN_MEANS:
        if (ef) MC_LAUNCH((sign_compress_k<SIGN_MEANS, true>), grid, block, lc, g, state_f, prev, beta, words, nwords, partial, hdr, algo);
        else MC_LAUNCH((sign_compress_k<SIGN_MEANS, false>), grid, block, lc, g, state_f, prev, beta, words, nwords, partial, hdr, algo);
        break;
    case SIGN_PLAIN:
        MC_LAUNCH((sign_compress_k<SIGN_PLAIN, false>), grid, block, lc, g, state_f, prev, beta, words, nwords, partial, hdr, algo);
        break;
    default:
        MC_LAUNCH((sign_compress_k<SIGN_MOMENTUM, true>), grid, block, lc, g, state_f, prev, beta, words, nwords, partial, hdr, algo);
        break;
    }
    prof_end(lc, K_EFSIGN_COMPRESS);
}

// ---------------------------------------------------------------------------
// One block: combine the per-block partials in a fixed order (bit-reproducible
// whatever the launch geometry of the producer was), derive the group scalar,
// write the payload header (and, for EF-Sign, the scale kept in the state).
//   RED_MEAN_ABS: scale = (float)(sum / n)      RED_L2: norm = (float)sqrt(sum)
//   RED_MAX_ABS : max of the partials (exact)   mode < 0: header only
//   RED_ONE     : scale = 1 (SignSGD, SigNUM: the decoded values are +-1)
//   RED_MEANS   : three partial arrays (sum of the upper class, of the lower class, size of the
//                 upper class) -> scale = mean of the upper class, second scalar = mean of the lower
// ---------------------------------------------------------------------------
constexpr int kFinalThreads = 1024;

__global__ __launch_bounds__(kFinalThreads) void scalar_finalize_k(const double *partial, uint32_t nblocks, int mode, uint32_t n,
                                                                   PayloadHeader *hdr, uint32_t algo, uint64_t k, uint32_t levels,
                                                                   float *state_scale)
{
    __shared__ double red[kFinalThreads / 64];
    if (mode == RED_MEANS) {
        // the three sums side by side (their loads in flight together, one barrier), each in the fixed order of the
        // single-sum case
        __shared__ double red3[3][kFinalThreads / 64];
        double acc3[3] = {0.0, 0.0, 0.0};
        for (uint32_t base = 0; base < nblocks; base += 8 * kFinalThreads) {
            double v[3][8];
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    uint32_t i = base + u * kFinalThreads + threadIdx.x;
                    v[a][u] = i < nblocks ? partial[(size_t)a * nblocks + i] : 0.0;
                }
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int u = 0; u < 8; ++u) acc3[a] += v[a][u];
        }
#pragma unroll
        for (int a = 0; a < 3; ++a) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) acc3[a] += __shfl_xor(acc3[a], m, 64);
            if ((threadIdx.x & 63) == 0) red3[a][threadIdx.x >> 6] = acc3[a];
        }
        __syncthreads();
        double S[3];
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            double T = red3[a][0];
            for (int w = 1; w < kFinalThreads / 64; ++w) T += red3[a][w];
            S[a] = T;
        }
        if (threadIdx.x == 0) {
            const double n_hi = S[2], n_lo = (double)n - S[2];
            const float hi = n_hi > 0.0 ? (float)(S[0] / n_hi) : 0.0f, lo = n_lo > 0.0 ? (float)(S[1] / n_lo) : 0.0f;
            PayloadHeader h;
            h.magic = kMagic; h.algo = algo; h.n = n; h.k = k; h.scale = hi; h.levels = levels;
            for (int i = 0; i < 24; ++i) h.pad[i] = 0;
            h.pad[0] = __float_as_uint(lo);
            *hdr = h;
            if (state_scale) { state_scale[0] = hi; state_scale[1] = lo; }
        }
        return;
    }
    double acc = 0.0;
    if (mode >= 0 && mode != RED_ONE) {
        // eight independent loads in flight per thread and round (one round up to 8192 partials);
        // the order of additions depends on nblocks only
        for (uint32_t base = 0; base < nblocks; base += 8 * kFinalThreads) {
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                uint32_t i = base + u * kFinalThreads + threadIdx.x;
                v[u] = i < nblocks ? partial[i] : 0.0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = mode == RED_MAX_ABS ? fmax(acc, v[u]) : acc + v[u];
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        double o = __shfl_xor(acc, m, 64);
        acc = mode == RED_MAX_ABS ? fmax(acc, o) : acc + o;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double S = red[0];
        for (int w = 1; w < kFinalThreads / 64; ++w) S = mode == RED_MAX_ABS ? fmax(S, red[w]) : S + red[w];
        float scale = 0.0f;
        if (n > 0) {
            if (mode == RED_MEAN_ABS) scale = (float)(S / (double)n);
            else if (mode == RED_L2) scale = (float)sqrt(S);
            else if (mode == RED_MAX_ABS) scale = (float)S;
        }
        if (mode == RED_ONE) scale = 1.0f;
        PayloadHeader h;
        h.magic = kMagic; h.algo = algo; h.n = n; h.k = k; h.scale = scale; h.levels = levels;
        for (int i = 0; i < 24; ++i) h.pad[i] = 0;
        *hdr = h;
        if (state_scale) *state_scale = scale;
    }
}

// state_scale: where the state keeps the scalar(s) of this call (EF-Sign: one float, OneBit: two), or null
void launch_scalar_finalize(const LaunchCtx &lc, const double *partial, uint32_t nblocks, int mode, uint32_t n,
                            PayloadHeader *hdr, uint32_t algo, uint64_t k, uint32_t levels, float *state_scale)
{
    prof_begin(lc, K_SCALAR_FINALIZE);
    MC_LAUNCH(scalar_finalize_k, dim3(1), dim3(kFinalThreads), lc, partial, nblocks, mode, n, hdr, algo, k,
                       levels, state_scale);
    prof_end(lc, K_SCALAR_FINALIZE);
}

// The two stochastic quantizers, one element: what is sent and what the receiver reconstructs from it.
// QSGD with a = |p| s / norm:  level = floor(a) + [u < a - floor(a)], code = sgn(p) level, d = code * (norm / s).
// The two per-group divisions are taken in fp64 and rounded once, which equals the correctly rounded
// fp32 quotient of two fp32 numbers.
struct QsgdScale {
    float norm, sf, r, q;
    int levels;
    __device__ __forceinline__ QsgdScale(float norm_, uint32_t levels_)
        : norm(norm_), sf((float)levels_), r(norm_ > 0.0f ? (float)((double)(float)levels_ / (double)norm_) : 0.0f),
          q((float)((double)norm_ / (double)(float)levels_)), levels((int)levels_) {}
};
__device__ __forceinline__ int qsgd_code(const QsgdScale &k, float p, float u)
{
    int xi = 0;
    if (k.norm > 0.0f) {
        // a >= s (or not a number) means level s: clamped to s, the steps below give exactly that (floor s, fraction 0,
        // and no u lies below 0), and below s the level cannot exceed s -- one minimum instead of a compare, a select
        // and a second clamp
        const float a = fminf(fabsf(p) * k.r, k.sf);
        const float l = floorf(a);
        const float f = a - l;
        xi = (int)l + (u < f ? 1 : 0);
    }
    return p < 0.0f ? -xi : xi;
}
__device__ __forceinline__ float qsgd_decode(const QsgdScale &k, int code) { return (float)code * k.q; }
// TernGrad: nz = [u * smax < |p|] (Bernoulli(|p| / smax) without a division), d = +-smax or 0
__device__ __forceinline__ float tern_decode(float smax, float p, float u, bool valid, bool &nz, bool &neg)
{
    nz = valid && (u * smax < fabsf(p));
    neg = nz && p < 0.0f;
    return nz ? (neg ? -smax : smax) : 0.0f;
}

// ---------------------------------------------------------------------------
// Pass A of the two-pass quantizers: p = g + e, kept in the state; per-block partial of
// sum p^2 (QSGD) or max |p| (TernGrad).
// The state never holds e itself: what pass B sends is a function of p, of the group
// scalar and of the random stream (worker, iteration) alone, so the residual of the last
// call is re-derived here as  e = p_prev - d(p_prev)  by quantizing p_prev again with the
// scalar and the stream that the state header recorded -- the same fp32 operations an
// explicit update would have used.  Pass B then writes no residual (17 instead of 21
// bytes per element over the two passes).  A zero-filled or imported state has scalar 0,
// for which d = 0 and e = p.
// ---------------------------------------------------------------------------
template <bool EF, int MODE>
__global__ __launch_bounds__(kBlock) void accum_reduce_k(GroupView g, float *st, const StateHeader *prev, uint32_t levels, uint64_t seed,
                                                         double *partial)
{
    __shared__ double red[kWavesPerBlock];
    __shared__ float redf[kWavesPerBlock];
    const Chunk c = my_chunk(g.n);
    double acc = 0.0;
    float mx = 0.0f;
    if (c.base < g.n) {
        float p[kSteps];
        load_seg(g, c, p);
        if (EF) {
            const float sprev = prev->scale;
            const uint32_t wprev = prev->prev_worker, iprev = prev->prev_iter;
            float q[kSteps], uni[kSteps];
            load_flat(st, c, g.n, q, 0.0f);
            chunk_uniforms(seed, wprev, iprev, g.goff + c.base, c.lane, uni);
            const QsgdScale ks(MODE == RED_L2 ? sprev : 0.0f, levels);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                float d;
                if (MODE == RED_L2) d = qsgd_decode(ks, qsgd_code(ks, q[j], uni[j]));
                else { bool nz, neg; d = tern_decode(sprev, q[j], uni[j], true, nz, neg); }
                const float e = q[j] - d;
                // past the end of the group there is nothing (QSGD with a subnormal norm decodes even a 0 to +-norm there)
                p[j] = c.full || c.base + 64 * j + c.lane < g.n ? p[j] + e : 0.0f;
            }
            store_flat(st, c, g.n, p);
        }
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {   // elements past n were loaded as 0 and add nothing
            if (MODE == RED_L2) acc += (double)p[j] * (double)p[j];
            else mx = fmaxf(mx, fabsf(p[j]));
        }
    }
    if (MODE == RED_L2) {
        double t = block_sum(acc, red);
        if (threadIdx.x == 0) partial[my_tile_index()] = t;
    } else {
        float t = block_max(mx, redf);
        if (threadIdx.x == 0) partial[my_tile_index()] = (double)t;
    }
}

void launch_accum_reduce(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, const StateHeader *prev, int mode,
                         uint32_t levels, uint64_t seed, double *partial)
{
    if (g.n == 0) return;
    dim3 grid(tiles_of(g.n)), block(kBlock);
    prof_begin(lc, K_ACCUM_REDUCE);
    if (mode == RED_L2) {
        if (ef) MC_LAUNCH((accum_reduce_k<true, RED_L2>), grid, block, lc, g, state_f, prev, levels, seed, partial);
        else MC_LAUNCH((accum_reduce_k<false, RED_L2>), grid, block, lc, g, state_f, prev, levels, seed, partial);
    } else {
        if (ef) MC_LAUNCH((accum_reduce_k<true, RED_MAX_ABS>), grid, block, lc, g, state_f, prev, levels, seed, partial);
        else MC_LAUNCH((accum_reduce_k<false, RED_MAX_ABS>), grid, block, lc, g, state_f, prev, levels, seed, partial);
    }
    prof_end(lc, K_ACCUM_REDUCE);
}

// p of pass B: from the state (where pass A left it) or, without error feedback, the gradient itself
template <bool EF>
__device__ __forceinline__ void load_p(const GroupView &g, const float *st, const Chunk &c, float (&p)[kSteps])
{
    if (EF) load_flat(st, c, g.n, p, 0.0f);
    else load_seg(g, c, p);
}

// Store one one-byte code per element of a chunk.  Codes are staged through LDS so that each lane
// writes 16 contiguous bytes (a wave store of 64 single bytes covers only half a cache line, and
// measured slower; the two-byte codes of FP16 cover a whole line and are stored directly).
template <typename T>
__device__ __forceinline__ void store_codes(T *codes, uint32_t n, uint32_t n_padded, const Chunk &c,
                                            const T (&v)[kSteps], T *stage /* kChunk entries, wave-private */)
{
    if (c.full) {
#pragma unroll
        for (int j = 0; j < kSteps; ++j) stage[64 * j + c.lane] = v[j];
        __builtin_amdgcn_wave_barrier();
        constexpr int kVec = (int)(kChunk * sizeof(T) / 16 / kWave);     // 16-byte vectors per lane
        const uint4 *src = reinterpret_cast<const uint4 *>(stage);
        uint4 *dst = reinterpret_cast<uint4 *>(codes + c.base);
#pragma unroll
        for (int r = 0; r < kVec; ++r) dst[r * 64 + c.lane] = src[r * 64 + c.lane];
        __builtin_amdgcn_wave_barrier();
    } else {
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            uint32_t i = c.base + 64 * j + c.lane;
            if (i < n) codes[i] = v[j];
            else if (i < n_padded) codes[i] = (T)0;      // zero padding up to a multiple of 4 bytes
        }
    }
}

// ---------------------------------------------------------------------------
// Pass B of the two-pass quantizers: the codes of p.  With error feedback p stays in the state
// as it is, and one thread records the group scalar and the random stream of this call in the
// state header, from which the next call's pass A re-derives the residual (see there).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void remember_call(StateHeader *sh, float scale, uint32_t worker, uint32_t iter_lo)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sh->scale = scale; sh->scale_lo = 0.0f; sh->prev_worker = worker; sh->prev_iter = iter_lo;
    }
}

template <bool EF>
__global__ __launch_bounds__(kBlock) void qsgd_encode_k(GroupView g, const float *st, StateHeader *sh, const PayloadHeader *hdr,
                                                        int8_t *codes, uint32_t levels, uint64_t seed, uint32_t worker, uint32_t iter_lo)
{
    __shared__ __attribute__((aligned(16))) int8_t stage[kWavesPerBlock][kChunk];
    const Chunk c = my_chunk(g.n);
    const float norm = hdr->scale;
    if (EF) remember_call(sh, norm, worker, iter_lo);
    if (c.base >= g.n) return;
    const QsgdScale ks(norm, levels);
    float p[kSteps];
    load_p<EF>(g, st, c, p);
    float uni[kSteps];
    chunk_uniforms(seed, worker, iter_lo, g.goff + c.base, c.lane, uni);
    int8_t code[kSteps];
#pragma unroll
    for (int j = 0; j < kSteps; ++j) code[j] = (int8_t)qsgd_code(ks, p[j], uni[j]);
    store_codes<int8_t>(codes, g.n, (g.n + 3u) & ~3u, c, code, stage[threadIdx.x >> 6]);
}

void launch_qsgd_encode(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, StateHeader *sh, const PayloadHeader *hdr,
                        int8_t *codes, uint32_t levels, uint64_t seed, uint32_t worker, uint32_t iter_lo)
{
    if (g.n == 0) return;
    dim3 grid(tiles_of(g.n)), block(kBlock);
    prof_begin(lc, K_QSGD_ENCODE);
    if (ef) MC_LAUNCH(qsgd_encode_k<true>, grid, block, lc, g, state_f, sh, hdr, codes, levels, seed, worker, iter_lo);
    else MC_LAUNCH(qsgd_encode_k<false>, grid, block, lc, g, state_f, sh, hdr, codes, levels, seed, worker, iter_lo);
    prof_end(lc, K_QSGD_ENCODE);
}

// TernGrad: two bit planes (non-zero, negative)
template <bool EF>
__global__ __launch_bounds__(kBlock) void tern_encode_k(GroupView g, const float *st, StateHeader *sh, const PayloadHeader *hdr,
                                                        uint32_t *planes, uint32_t nwords, uint64_t seed, uint32_t worker, uint32_t iter_lo)
{
    __shared__ uint64_t stage[kWavesPerBlock][kSteps];
    const Chunk c = my_chunk(g.n);
    const float smax = hdr->scale;
    if (EF) remember_call(sh, smax, worker, iter_lo);
    if (c.base >= g.n) return;
    float p[kSteps];
    load_p<EF>(g, st, c, p);
    float uni[kSteps];
    chunk_uniforms(seed, worker, iter_lo, g.goff + c.base, c.lane, uni);
    uint64_t bnz[kSteps], bng[kSteps];
#pragma unroll
    for (int j = 0; j < kSteps; ++j) {
        uint32_t i = c.base + 64 * j + c.lane;
        bool valid = c.full || i < g.n;
        bool nz, neg;
        (void)tern_decode(smax, p[j], uni[j], valid, nz, neg);
        bnz[j] = __builtin_amdgcn_ballot_w64(nz);
        bng[j] = __builtin_amdgcn_ballot_w64(neg);
    }
    store_plane(planes, nwords, c, bnz, stage[threadIdx.x >> 6]);
    store_plane(planes + nwords, nwords, c, bng, stage[threadIdx.x >> 6]);
}

void launch_tern_encode(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, StateHeader *sh, const PayloadHeader *hdr,
                        uint32_t *planes, uint32_t nwords, uint64_t seed, uint32_t worker, uint32_t iter_lo)
{
    if (g.n == 0) return;
    dim3 grid(tiles_of(g.n)), block(kBlock);
    prof_begin(lc, K_TERN_ENCODE);
    if (ef) MC_LAUNCH(tern_encode_k<true>, grid, block, lc, g, state_f, sh, hdr, planes, nwords, seed, worker, iter_lo);
    else MC_LAUNCH(tern_encode_k<false>, grid, block, lc, g, state_f, sh, hdr, planes, nwords, seed, worker, iter_lo);
    prof_end(lc, K_TERN_ENCODE);
}

// ---------------------------------------------------------------------------
// FP16, single pass: h = binary16(p) round-to-nearest-even, e <- p - (float)h.
// ---------------------------------------------------------------------------
template <bool EF>
__global__ __launch_bounds__(kBlock) void fp16_compress_k(GroupView g, float *st, uint16_t *halves, PayloadHeader *hdr)
{
    const Chunk c = my_chunk(g.n);
    if (blockIdx.x == 0 && threadIdx.x == 0) put_plain_header(hdr, MC_ALGO_FP16, g.n, 0.0f);
    if (c.base >= g.n) return;
    float p[kSteps];
    load_seg(g, c, p);
    if (EF) {
        float e[kSteps];
        load_flat(st, c, g.n, e, 0.0f);
#pragma unroll
        for (int j = 0; j < kSteps; ++j) p[j] = p[j] + e[j];
    }
    uint16_t h[kSteps];
    float e[kSteps];
#pragma unroll
    for (int j = 0; j < kSteps; ++j) {
        _Float16 hv = (_Float16)p[j];                 // v_cvt_f16_f32: round to nearest even, keeps subnormals
        h[j] = __builtin_bit_cast(uint16_t, hv);
        e[j] = p[j] - (float)hv;
    }
    if (EF) store_flat(st, c, g.n, e);
    // 64 lanes x 2 bytes: one whole 128-byte line per wave store (the body of a payload starts on a line), which
    // measured faster than 16-byte stores out of an LDS stage (58.6 against 65.0 us for the kernel's call)
    if (c.full) {
        uint16_t *dst = halves + c.base + c.lane;
#pragma unroll
        for (int j = 0; j < kSteps; ++j) st_stream(dst + 64 * j, h[j]);
    } else {
        const uint32_t n_padded = (g.n + 1u) & ~1u;       // zero padding up to a multiple of 4 bytes
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            const uint32_t i = c.base + 64 * j + c.lane;
            if (i < g.n) halves[i] = h[j];
            else if (i < n_padded) halves[i] = (uint16_t)0;
        }
    }
}

void launch_fp16_compress(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, PayloadHeader *hdr,
                          uint16_t *halves)
{
    if (g.n == 0) return;
    dim3 grid(tiles_of(g.n)), block(kBlock);
    prof_begin(lc, K_FP16_COMPRESS);
    if (ef) MC_LAUNCH(fp16_compress_k<true>, grid, block, lc, g, state_f, halves, hdr);
    else MC_LAUNCH(fp16_compress_k<false>, grid, block, lc, g, state_f, halves, hdr);
    prof_end(lc, K_FP16_COMPRESS);
}

// ---------------------------------------------------------------------------
// Decompress-and-sum of dense codes (Algorithm 1: g~ = aggregate(C^-1(Delta))):
// out_i = alpha * (((0 + d_0,i) + d_1,i) + ...), workers in ascending order, one
// pass, every payload read once, the dense result written once through the
// segment table.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void check_header(const PayloadHeader *h, uint32_t algo, uint32_t n, int *status)
{
    if (h->magic != kMagic || h->algo != algo || h->n != (uint64_t)n) *status = 1;
}

// Workers are taken in batches: all loads of a batch (header scalars and codes)
// are issued before the first is used, so a wavefront pays the HBM latency once
// per batch instead of once per worker.
//
// Two lane mappings.  Wide (QSGD, a full chunk inside one tensor whose address is 16-byte aligned):
// lane l holds four consecutive elements in each of four steps, element (256 m + 4 l + rot) mod 1024
// onward, so the codes of a worker arrive in 4 loads of 4 bytes per lane instead of 16 loads of one
// byte, and the sums leave as 16-byte stores; rot puts the stores on the output's 128-byte lines.
// Plain (FP16, and any other chunk): the usual element 64 j + l per step.  The work is elementwise,
// so the mapping changes no result: every element still adds its workers' values in worker order.
// (Measured, 8 workers, 25.6 M elements: QSGD 62.9 -> 54.6 us.  The same mapping with 8-byte loads
// made FP16 slower, 80.3 -> 82.5..85 us with 2, 4 or 8 workers per batch, so FP16 stays plain.)
typedef float float4v __attribute__((ext_vector_type(4)));

template <int ALGO>
__global__ __launch_bounds__(kBlock) void dense_decompress_k(GroupView out, PayloadPtrs pl, int W, float alpha,
                                                             uint32_t levels, int *status)
{
    static_assert(ALGO == MC_ALGO_QSGD || ALGO == MC_ALGO_FP16, "one code per element");
    constexpr int kBatch = 4;
    const Chunk c = my_chunk(out.n);
    if (blockIdx.x == 0 && (int)threadIdx.x < W)
        check_header(reinterpret_cast<const PayloadHeader *>(pl.p[threadIdx.x]), ALGO, out.n, status);
    if (c.base >= out.n) return;
    const uintptr_t entry = chunk_entry(out, c);
    if (ALGO == MC_ALGO_QSGD && !(entry & 15u)) {               // an address (even), and 16-byte aligned
        const uint32_t rot = chunk_rotation(entry);             // a multiple of 4 here
        uint32_t at[4];                                         // first of the lane's four elements in step m
#pragma unroll
        for (int m = 0; m < 4; ++m) at[m] = (256u * m + 4u * c.lane + rot) & (uint32_t)(kChunk - 1);
        float acc[4][4];
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[m][e] = 0.0f;
        for (int w0 = 0; w0 < W; w0 += kBatch) {
            float scale[kBatch];
#pragma unroll
            for (int b = 0; b < kBatch; ++b)
                scale[b] = w0 + b < W ? ld_uniform(&reinterpret_cast<const PayloadHeader *>(pl.p[w0 + b])->scale) : 0.0f;
            uint32_t cw[kBatch][4];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const uint8_t *codes = pl.p[w0 + b < W ? w0 + b : 0] + kHeaderBytes + c.base;
#pragma unroll
                for (int m = 0; m < 4; ++m) cw[b][m] = w0 + b < W ? ld_stream(reinterpret_cast<const uint32_t *>(codes + at[m])) : 0u;
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                if (w0 + b < W) {
                    const float q = (float)((double)scale[b] / (double)(float)levels);
#pragma unroll
                    for (int m = 0; m < 4; ++m)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[m][e] = acc[m][e] + (float)(int8_t)(cw[b][m] >> (8 * e)) * q;
                }
            }
        }
        float *p = reinterpret_cast<float *>(entry);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            float4v v = {alpha * acc[m][0], alpha * acc[m][1], alpha * acc[m][2], alpha * acc[m][3]};
            __builtin_nontemporal_store(v, reinterpret_cast<float4v *>(p + at[m]));
        }
        return;
    }
    float acc[kSteps];
#pragma unroll
    for (int j = 0; j < kSteps; ++j) acc[j] = 0.0f;
    for (int w0 = 0; w0 < W; w0 += kBatch) {
        float scale[kBatch];
#pragma unroll
        for (int b = 0; b < kBatch; ++b)
            scale[b] = w0 + b < W ? ld_uniform(&reinterpret_cast<const PayloadHeader *>(pl.p[w0 + b])->scale) : 0.0f;
        if (ALGO == MC_ALGO_QSGD) {
            int8_t cd[kBatch][kSteps];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                if (w0 + b < W) load_flat<int8_t>(reinterpret_cast<const int8_t *>(pl.p[w0 + b] + kHeaderBytes), c, out.n, cd[b], (int8_t)0);
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                if (w0 + b < W) {
                    const float q = (float)((double)scale[b] / (double)(float)levels);
#pragma unroll
                    for (int j = 0; j < kSteps; ++j) acc[j] = acc[j] + (float)cd[b][j] * q;
                }
            }
        } else {   // FP16
            _Float16 hv[kBatch][kSteps];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                if (w0 + b < W) load_flat<_Float16>(reinterpret_cast<const _Float16 *>(pl.p[w0 + b] + kHeaderBytes), c, out.n, hv[b], (_Float16)0.0f);
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                if (w0 + b < W) {
#pragma unroll
                    for (int j = 0; j < kSteps; ++j) acc[j] = acc[j] + (float)hv[b][j];
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kSteps; ++j) acc[j] = alpha * acc[j];
    store_seg(out, c, acc, entry);
}

// ---------------------------------------------------------------------------
// EF-Sign / TernGrad decompress-and-sum.  With W sign planes the per-element work of the
// generic kernel (extract bit, select +-scale, add; W times) exceeds what the
// vector ALUs can do at HBM speed, so this kernel works on whole words:
//   * the sum of the first (up to) 8 workers takes one of 2^8 values per group;
//     every block tabulates them in LDS with the very same sequence of fp32
//     additions  ((0 + d_0) + d_1) + ... , so a lookup returns the exact result;
//   * a lane owns 32 consecutive elements, i.e. one word of every worker's plane;
//     four 8x8 bit-matrix transposes turn its 8 words into 32 table indices;
//   * further workers (W > 8) are added one by one in order;
//   * results go through a skewed LDS stage so that the global stores are the
//     usual 256 contiguous bytes per wave instruction.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t transpose8x8(uint64_t x)
{
    // bit (8 r + c) <-> bit (8 c + r): three rounds of masked swaps
    uint64_t t;
    t = 0x0f0f0f0f00000000ull & (x ^ (x << 28)); x ^= t ^ (t >> 28);
    t = 0x3333000033330000ull & (x ^ (x << 14)); x ^= t ^ (t >> 14);
    t = 0x5500550055005500ull & (x ^ (x << 7));  x ^= t ^ (t >> 7);
    return x;
}

constexpr int kSignWaveElems = 2048;                       // 64 lanes x 32 elements
constexpr int kSignTile = kSignWaveElems * kWavesPerBlock; // 8192 elements per block

// bytes of 8 words (one per worker) -> per element the 8 workers' bits: word q byte -> 8 table indices
__device__ __forceinline__ uint64_t gather_transpose(const uint32_t (&wd)[8], int q)
{
    uint32_t lo = ((wd[0] >> (8 * q)) & 0xFFu) | (((wd[1] >> (8 * q)) & 0xFFu) << 8) |
                  (((wd[2] >> (8 * q)) & 0xFFu) << 16) | (((wd[3] >> (8 * q)) & 0xFFu) << 24);
    uint32_t hi = ((wd[4] >> (8 * q)) & 0xFFu) | (((wd[5] >> (8 * q)) & 0xFFu) << 8) |
                  (((wd[6] >> (8 * q)) & 0xFFu) << 16) | (((wd[7] >> (8 * q)) & 0xFFu) << 24);
    return transpose8x8((uint64_t)lo | ((uint64_t)hi << 32));
}

// TERN = false: the one-plane schemes (2^8 sums of the first 8 workers' +-level).  TERN = true: TernGrad
// (non-zero and negative planes; a worker contributes 0, +s or -s): the table holds the 2^8 possible sums
// of workers 0..3, indexed by their four non-zero and four negative bits, and workers 4..7 are added one
// by one, so that every element sees the sequence of fp32 additions ((0 + d_0) + d_1) + ... of a plain
// loop.  (A table of all 3^8 sums of 8 workers needs 26 KB of LDS per block and a kernel of its own to
// fill it, and measured slower; a second table over workers 0..5, 4096 entries filled from the first,
// 35.5 against 36.0 us.)
// what a set / clear bit of worker w decodes to (one-plane schemes)
__device__ __forceinline__ void plane_levels(const PayloadHeader *h, int kind, float &hi, float &lo)
{
    // (scalar loads: as vector loads they queue behind the compute unit's stores, and every block waits for them)
    hi = kind == PLANE_VOTE ? 1.0f : ld_uniform(&h->scale);
    lo = kind == PLANE_MEANS ? __uint_as_float(ld_uniform(&h->pad[0])) : -hi;
}
__device__ __forceinline__ float vote_of(float tally) { return tally > 0.0f ? 1.0f : (tally < 0.0f ? -1.0f : 0.0f); }

// kind (one-plane schemes only): PLANE_SCALE  EF-Sign, a bit decodes to +-scale
//                                PLANE_MEANS  OneBit, to the mean of its class
//                                PLANE_VOTE   SignSGD / SigNUM, to +-1, and the sum becomes its sign (majority vote)
// Bit e of a TernGrad worker's two plane words -> what the worker adds to element e: 0, +s or -s, as bit
// operations on s (a one-bit field, sign-extended, is the mask).  The masks pass through an empty asm so that the
// compiler does not turn them back into compares and selects (9 issue slots with their wait states instead of 5).
__device__ __forceinline__ float tern_term(uint32_t nzw, uint32_t ngw, int e, float sc)
{
    uint32_t mx = (uint32_t)__builtin_amdgcn_sbfe((int)nzw, e, 1), my = (uint32_t)__builtin_amdgcn_sbfe((int)ngw, e, 1);
    asm("" : "+v"(mx));
    asm("" : "+v"(my));
    return __uint_as_float((__float_as_uint(sc) ^ (my & 0x80000000u)) & mx);
}

// bit e of a one-plane worker's word -> the level it decodes to, the same way
__device__ __forceinline__ float plane_term(uint32_t word, int e, float hi, float lo)
{
    uint32_t m = (uint32_t)__builtin_amdgcn_sbfe((int)word, e, 1);
    asm("" : "+v"(m));
    return __uint_as_float((__float_as_uint(hi) & m) | (__float_as_uint(lo) & ~m));
}

template <bool TERN>
__global__ __launch_bounds__(kBlock) void plane_decompress_k(GroupView out, PayloadPtrs pl, int W, float alpha, int *status,
                                                             int algo, int kind)
{
    __shared__ float table[256];
    __shared__ float stage[kWavesPerBlock][kChunk + 32];
    const uint32_t t = threadIdx.x;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63u;
    if (blockIdx.x == 0 && (int)t < W)
        check_header(reinterpret_cast<const PayloadHeader *>(pl.p[t]), algo, out.n, status);
    const int Wt = W < 8 ? W : 8;
    // the plane words are asked for before the table is built: the headers' scalars, which the table waits for, and
    // the words then travel together (one-plane schemes 0.6 us, OneBit and TernGrad 1.0-1.5 us of 28-37)
    const uint32_t wbase = my_tile_index() * (uint32_t)kSignTile + wave * (uint32_t)kSignWaveElems;
    const uint32_t nwords = (out.n + 31u) >> 5;
    const uint32_t wi = (wbase >> 5) + lane;
    uint32_t wd[8], wn[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        wd[b] = 0u; wn[b] = 0u;
        if (b < Wt && wi < nwords) {
            const uint32_t *plane = reinterpret_cast<const uint32_t *>(pl.p[b] + kHeaderBytes);
            wd[b] = ld_stream(plane + wi);
            if (TERN) wn[b] = ld_stream(plane + nwords + wi);
        }
    }
    {
        if (!TERN) {
            float acc = 0.0f;
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                if (b < Wt) {
                    float hi, lo;
                    plane_levels(reinterpret_cast<const PayloadHeader *>(pl.p[b]), kind, hi, lo);
                    acc = acc + (((t >> b) & 1u) ? hi : lo);
                }
            }
            if (W <= 8 && kind == PLANE_VOTE) acc = vote_of(acc);
            table[t] = W <= 8 ? alpha * acc : acc;
        } else {
            // entry (nz bits of workers 0..3) | (negative bits of workers 0..3) << 4: their sum, in worker order
            float acc = 0.0f;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (b < Wt) {
                    const float sc = ld_uniform(&reinterpret_cast<const PayloadHeader *>(pl.p[b])->scale);
                    acc = acc + (((t >> b) & 1u) ? (((t >> (4 + b)) & 1u) ? -sc : sc) : 0.0f);
                }
            }
            table[t] = acc;
        }
    }
    float s47[4] = {0.0f, 0.0f, 0.0f, 0.0f};               // TernGrad: scales of workers 4..7, added one by one
    if (TERN) {
#pragma unroll
        for (int b = 4; b < 8; ++b) if (b < Wt) s47[b - 4] = ld_uniform(&reinterpret_cast<const PayloadHeader *>(pl.p[b])->scale);
    }
    __syncthreads();
    if (wbase >= out.n) return;
    float acc[32];
    // TernGrad: only workers 0..3 enter the transposes
    const uint32_t wlow[8] = {wd[0], wd[1], wd[2], wd[3], 0u, 0u, 0u, 0u}, nlow[8] = {wn[0], wn[1], wn[2], wn[3], 0u, 0u, 0u, 0u};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // byte q of the 8 words -> rows of an 8x8 bit matrix (row = worker, column = element 8q + c)
        const uint64_t x = TERN ? gather_transpose(wlow, q) : gather_transpose(wd, q);
        if (!TERN) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[8 * q + e] = table[(uint32_t)(x >> (8 * e)) & 0xFFu];
        } else {
            // workers 0..3 through the table (their bits transposed into an index), workers 4..7 straight from their
            // words.  An absent worker (W < 8: words and scale 0) adds +0, which changes no sum: none is ever -0.
            const uint64_t y = gather_transpose(nlow, q) & x;         // negative only counts where non-zero
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t xe = (uint32_t)(x >> (8 * e)) & 15u, ye = (uint32_t)(y >> (8 * e)) & 15u;
                float a = table[xe | (ye << 4)];
#pragma unroll
                for (int b = 4; b < 8; ++b) a = a + tern_term(wd[b], wn[b], 8 * q + e, s47[b - 4]);
                acc[8 * q + e] = a;
            }
        }
    }
    if (W > 8) {
        for (int w = 8; w < W; ++w) {
            float sc = ld_uniform(&reinterpret_cast<const PayloadHeader *>(pl.p[w])->scale), sl = -sc;
            if (!TERN) plane_levels(reinterpret_cast<const PayloadHeader *>(pl.p[w]), kind, sc, sl);
            const uint32_t *plane = reinterpret_cast<const uint32_t *>(pl.p[w] + kHeaderBytes);
            const uint32_t word = wi < nwords ? ld_stream(plane + wi) : 0u;
            const uint32_t neg = TERN && wi < nwords ? ld_stream(plane + nwords + wi) : 0u;
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                float d;
                if (!TERN) d = plane_term(word, e, sc, sl);
                else d = tern_term(word, neg, e, sc);
                acc[e] = acc[e] + d;
            }
        }
    }
    if (W > 8 || TERN) {
#pragma unroll
        for (int e = 0; e < 32; ++e) acc[e] = alpha * (!TERN && kind == PLANE_VOTE ? vote_of(acc[e]) : acc[e]);
    }
    // two halves of 1024 elements through one skewed LDS stage (lanes 32 h .. 32 h + 31 own the elements of
    // half h), so that the global stores are 256 contiguous bytes per wave instruction
    float *mine = stage[wave];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        __builtin_amdgcn_wave_barrier();
        if ((lane >> 5) == (uint32_t)half) {
#pragma unroll
            for (int e = 0; e < 32; ++e) mine[33 * (lane & 31u) + e] = acc[e];     // element 32 (lane % 32) + e, skewed
        }
        __builtin_amdgcn_wave_barrier();
        Chunk c;
        c.base = wbase + half * (uint32_t)kChunk;
        c.lane = lane;
        c.full = c.base < out.n && out.n - c.base >= (uint32_t)kChunk;
        if (c.base < out.n) {
            const uintptr_t entry = chunk_entry(out, c);
            const uint32_t rot = TERN ? 0u : chunk_rotation(entry);     // measured: no gain for TernGrad, whose decode is bound by the vector ALU
            float v[kSteps];
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                const uint32_t i = rotated(j, lane, rot);                // element of this half, rotated onto the lines
                v[j] = mine[i + (i >> 5)];
            }
            store_seg_rot(out, c, v, entry, rot);
        }
    }
}

void launch_dense_decompress(const LaunchCtx &lc, int algo, const GroupView &out, const PayloadPtrs &pl, int W,
                             float alpha, uint32_t levels, int *status)
{
    if (out.n == 0) return;
    dim3 grid(tiles_of(out.n)), block(kBlock);
    prof_begin(lc, K_DENSE_DECOMPRESS);
    switch (algo) {
    case MC_ALGO_EFSIGN:
    case MC_ALGO_ONEBIT:
    case MC_ALGO_SIGNSGD:
    case MC_ALGO_SIGNUM:
        MC_LAUNCH(plane_decompress_k<false>, dim3((uint32_t)(((uint64_t)out.n + kSignTile - 1) / kSignTile)), block, lc, out, pl, W,
                  alpha, status, algo,
                  algo == MC_ALGO_EFSIGN ? PLANE_SCALE : algo == MC_ALGO_ONEBIT ? PLANE_MEANS : PLANE_VOTE);
        break;
    case MC_ALGO_TERNGRAD:
        MC_LAUNCH(plane_decompress_k<true>, dim3((uint32_t)(((uint64_t)out.n + kSignTile - 1) / kSignTile)), block, lc, out, pl, W,
                  alpha, status, algo, PLANE_SCALE);
        break;
    case MC_ALGO_QSGD: MC_LAUNCH(dense_decompress_k<MC_ALGO_QSGD>, grid, block, lc, out, pl, W, alpha, levels, status); break;
    default: MC_LAUNCH(dense_decompress_k<MC_ALGO_FP16>, grid, block, lc, out, pl, W, alpha, levels, status); break;
    }
    prof_end(lc, K_DENSE_DECOMPRESS);
}

// ---------------------------------------------------------------------------
// State <-> plain residual.  EF-Sign, OneBit, QSGD and TernGrad keep p and the scalars
// of the last call instead of the residual; the other algorithms copy (SigNUM: the momentum).
// ---------------------------------------------------------------------------
// One thread per element of the group (a launch holds fewer than 2^32 threads, and DGC's two vectors together
// may hold more floats than that): the thread of element i converts float i of every vector.
__global__ __launch_bounds__(kBlock) void state_convert_k(int algo, int to_residual, uint32_t n, const uint8_t *src, uint8_t *dst,
                                                          uint32_t levels, uint64_t seed, uint64_t goff)
{
    // plain side: n floats (DGC: v[n] then u[n]); opaque side: header, then the same floats (DGC: u from dgc_u_offset(n))
    const size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    const size_t uoff = dgc_u_offset(n);
    if (to_residual) {
        const StateHeader *h = reinterpret_cast<const StateHeader *>(src);
        const float *f = reinterpret_cast<const float *>(src + kHeaderBytes);
        float *e = reinterpret_cast<float *>(dst);
        if (i < n) {
            float v = f[i];
            if (algo == MC_ALGO_EFSIGN) { float sp = h->scale; v = v - (v >= 0.0f ? sp : -sp); }
            if (algo == MC_ALGO_ONEBIT) v = v - (v >= 0.0f ? h->scale : h->scale_lo);
            if (algo == MC_ALGO_QSGD || algo == MC_ALGO_TERNGRAD) {
                // what the last call sent of p is quantized once more, with its scalar and its random stream
                uint32_t w[4];
                philox4x32_10(seed, h->prev_worker, h->prev_iter, (goff + i) >> 2, w);
                const uint32_t word = (goff + i) & 3u;
                const float u = u01(word == 0 ? w[0] : word == 1 ? w[1] : word == 2 ? w[2] : w[3]);
                float d;
                if (algo == MC_ALGO_QSGD) { const QsgdScale ks(h->scale, levels); d = qsgd_decode(ks, qsgd_code(ks, v, u)); }
                else { bool nz, neg; d = tern_decode(h->scale, v, u, true, nz, neg); }
                v = v - d;
            }
            // Top-k, DGC: what the last call sent above its threshold key is masked by the next streaming pass, not zeroed
            const bool sent = (algo == MC_ALGO_TOPK || algo == MC_ALGO_DGC) && (__float_as_uint(v) & 0x7FFFFFFFu) > h->sent_key;
            e[i] = sent ? 0.0f : v;
            if (algo == MC_ALGO_DGC) e[(size_t)n + i] = sent ? 0.0f : f[uoff + i];
        }
    } else {
        const float *e = reinterpret_cast<const float *>(src);
        float *f = reinterpret_cast<float *>(dst + kHeaderBytes);
        if (i < n) {
            f[i] = e[i];                      // EF-Sign, OneBit, QSGD, TernGrad: p = e with scalars 0 re-derives exactly e
            if (algo == MC_ALGO_DGC) f[uoff + i] = e[(size_t)n + i];
        }
        // a cleared header; for the sparsifiers sent_key = all ones: nothing of an imported residual counts as sent
        if (i < kHeaderBytes / 4)
            reinterpret_cast<uint32_t *>(dst)[i] = i == offsetof(StateHeader, sent_key) / 4 && (algo == MC_ALGO_TOPK || algo == MC_ALGO_DGC || algo == MC_ALGO_RANDK) ? 0xFFFFFFFFu : 0u;
        if (algo == MC_ALGO_DGC && i >= n && i < uoff) f[i] = 0.0f;                       // the gap between v and u
    }
}

void launch_state_convert(const LaunchCtx &lc, int algo, bool to_residual, uint32_t n, const void *src, void *dst, uint32_t levels,
                          uint64_t seed, uint64_t goff)
{
    // the header is cleared too, and so is DGC's gap (fewer than 32 floats past n)
    const size_t work = (size_t)n + 32u > (size_t)kHeaderBytes / 4 ? (size_t)n + 32u : (size_t)kHeaderBytes / 4;
    prof_begin(lc, K_STATE_CONVERT);
    MC_LAUNCH(state_convert_k, dim3((uint32_t)((work + kBlock - 1) / kBlock)), dim3(kBlock), lc, algo,
                       to_residual ? 1 : 0, n, (const uint8_t *)src, (uint8_t *)dst, levels, seed, goff);
    prof_end(lc, K_STATE_CONVERT);
}

}  // namespace mc
