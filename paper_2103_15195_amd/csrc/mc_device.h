// Device-side building blocks shared by the gfx950 kernels: the wave-chunk
// element mapping, segment-table addressing, reductions and Philox.
//
// Element mapping.  A block of 256 threads (4 wavefronts of 64) owns a tile of
// 4096 consecutive flat elements of a merged group; wavefront w owns the
// 1024-element chunk starting at tile + 1024 w, and in step j (0..15) lane l
// holds flat element  chunk + 64 j + l.  A wave instruction therefore touches 256
// contiguous bytes whatever the alignment of the tensors behind the flat index,
// and a 64-bit ballot of step j is exactly two consecutive 32-bit words of a
// packed bit plane.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mc {

constexpr int kBlock = 256;
constexpr int kWave = 64;
constexpr int kSteps = 16;                  // elements per lane per chunk
constexpr int kChunk = kWave * kSteps;      // 1024 elements per wavefront
constexpr int kTile = kBlock * kSteps;      // 4096 elements per block
constexpr int kWavesPerBlock = kBlock / kWave;

// A merged group as the kernels see it: the flat index space [0, n) laid over
// `nseg` non-empty tensors.  seg_off[s] is the flat index of the first element
// of tensor s (strictly increasing, seg_off[nseg] = n); ptrs[s] its address.
struct GroupView {
    const uint32_t *seg_off;
    const uint32_t *chunk_seg;   // tensor that holds the first element of each 1024-element chunk
    const uintptr_t *ptrs;
    const uintptr_t *chunk_addr; // per chunk: its address if the whole chunk lies in one tensor, else 2 * first tensor + 1 (chunk_entry)
    uint32_t nseg;
    uint32_t n;
    uint64_t goff;   // model-global flat index of element 0 (random streams only)
};

struct Chunk {
    uint32_t base;   // flat index of the chunk's first element (wave-uniform)
    uint32_t lane;
    bool full;       // the whole chunk lies below n
};

// Tiles are handed out last first (block 0 takes the last tile).  The chunks that straddle tensors are the slow
// ones, and in a model's gradient list they crowd where the small tensors are -- at the end, when the list is in
// the order the gradients become ready, the first layers last.  Started first, they are hidden behind the rest
// (read-only pass over the ResNet-50 list: 18.0 us instead of 19.5; 17.1 with no such chunk at all).
__device__ __forceinline__ uint32_t my_tile_index() { return gridDim.x - 1u - blockIdx.x; }

__device__ __forceinline__ Chunk my_chunk(uint32_t n, uint32_t tile)
{
    Chunk c;
    uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.base = tile * (uint32_t)kTile + wave * (uint32_t)kChunk;
    c.lane = threadIdx.x & 63u;
    c.full = c.base < n && n - c.base >= (uint32_t)kChunk;
    return c;
}
__device__ __forceinline__ Chunk my_chunk(uint32_t n) { return my_chunk(n, my_tile_index()); }

// A load whose address is the same for the whole wavefront, forced onto the scalar path (constant address
// space).  In a kernel that streams stores, loads on the vector path queue behind those stores; the scalar
// cache does not.  (Measured: the same 16 table loads per wavefront cost the sparse decompress 5-7 us more
// when the compiler happened to issue them as vector loads.)  Only for data no thread of this kernel writes.
template <typename T>
__device__ __forceinline__ T ld_uniform(const T *p)
{
    typedef const T __attribute__((address_space(4))) *const_ptr;
    return *(const_ptr)(uintptr_t)p;
}

template <typename T>
__device__ __forceinline__ T ld_stream(const T *p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ __forceinline__ void st_stream(T *p, T v) { __builtin_nontemporal_store(v, p); }

// ---- flat (contiguous) buffers -------------------------------------------
template <typename T>
__device__ __forceinline__ void load_flat(const T *buf, const Chunk &c, uint32_t n, T (&v)[kSteps], T fill)
{
    const T *p = buf + c.base + c.lane;
    if (c.full) {
#pragma unroll
        for (int j = 0; j < kSteps; ++j) v[j] = ld_stream(p + 64 * j);
    } else {
#pragma unroll
        for (int j = 0; j < kSteps; ++j) v[j] = (c.base + 64 * j + c.lane < n) ? p[64 * j] : fill;
    }
}

template <typename T>
__device__ __forceinline__ void store_flat(T *buf, const Chunk &c, uint32_t n, const T (&v)[kSteps])
{
    T *p = buf + c.base + c.lane;
    if (c.full) {
#pragma unroll
        for (int j = 0; j < kSteps; ++j) st_stream(p + 64 * j, v[j]);
    } else {
#pragma unroll
        for (int j = 0; j < kSteps; ++j) if (c.base + 64 * j + c.lane < n) p[64 * j] = v[j];
    }
}

// ---- rotated chunks ----------------------------------------------------------
// Stores are sensitive to where a wave instruction's 256 bytes start: on this part the plane decompress
// kernel takes 27 us when they start on 128-byte lines, 32 us when they are 32 bytes off (separately
// allocated tensors whose sizes are not multiples of 32 elements put every chunk of the flat grid off the
// lines), and 30.4 us when they only start on 64-byte boundaries.  A kernel that takes its output from
// LDS may permute a chunk's elements among its lanes freely, so it can rotate the mapping by `rot`
// elements: in step j lane l holds element (64 j + l + rot) mod 1024 of the chunk, with rot chosen such
// that element `rot` lies on a line boundary.  Every wave store then covers two whole lines; only step 15
// wraps round to the chunk's first `rot` elements.  (Measured in the library: the one-plane decompress
// gains 2.4-3 us of 32 and the sparse decompress 0.5 us on its zero-fill path; the TernGrad decompress and
// the sparse one's LDS path lose 1.5-3 us, QSGD and FP16 lose up to 8 us when their code loads are rotated
// too (they then straddle lines) and gain or lose about 1 us when only the sums are rotated with
// ds_bpermute: those keep the plain mapping.)
constexpr uint32_t kLineElems = 32;        // 128-byte cache line
__device__ __forceinline__ uint32_t chunk_rotation(uintptr_t entry)       // 0 for a chunk without an address of its own
{
    return (entry & 1u) ? 0u : (kLineElems - (uint32_t)((entry >> 2) & (kLineElems - 1u))) & (kLineElems - 1u);
}
__device__ __forceinline__ uint32_t rotated(int j, uint32_t lane, uint32_t rot)
{
    const uint32_t i = 64u * (uint32_t)j + lane + rot;       // below 1024 except, possibly, in the last step
    return j == kSteps - 1 ? i & (uint32_t)(kChunk - 1) : i;
}

// The per-chunk table entry: the address of the chunk's first element when all 1024 elements lie in one
// tensor (even: tensors are 4-byte aligned), else 2 s + 1 with s the tensor that holds the chunk's first
// element (where the loop over the chunk's tensors starts).  Never 0.  A kernel that has other loads to
// wait for before it stores fetches this first, so that the two latencies overlap.
__device__ __forceinline__ uintptr_t chunk_entry(const GroupView &g, const Chunk &c) { return ld_uniform(g.chunk_addr + (c.base >> 10)); }

// ---- segmented (per-tensor) buffers ------------------------------------------
// Fast path: the chunk lies inside one tensor and its address was tabulated when
// the tensor address list was uploaded (one scalar load, then the data).
// Otherwise (the chunk straddles tensors, or is the ragged last one) the wavefront
// fetches the table entries of up to 64 tensors from the chunk's first one on, one per
// lane, and then takes the tensors one by one -- a wave-uniform loop whose bounds and
// addresses come out of the lanes -- so that the data accesses wait for one round of
// table loads only.  (A per-lane walk of the table, two dependent loads per tensor
// boundary, made the ~100 such chunks of the ResNet-50 list the last to finish: 21
// instead of 17 us for a read-only pass over the 102 MB.)
template <typename Body>
__device__ __forceinline__ void for_each_tensor_of_chunk(const GroupView &g, const Chunk &c, uint32_t s0, Body body)
{
    const uint32_t lim = g.n - c.base >= (uint32_t)kChunk ? c.base + (uint32_t)kChunk : g.n;     // end of the chunk
    for (;;) {
        const uint32_t t = s0 + c.lane;
        const uint32_t beg = g.seg_off[t < g.nseg ? t : g.nseg];                 // seg_off has nseg + 1 entries, the last is n
        const uint32_t end = g.seg_off[t < g.nseg ? t + 1u : g.nseg];
        const uintptr_t ptr = g.ptrs[t < g.nseg ? t : g.nseg - 1u];
        for (int k = 0; k < 64; ++k) {
            const uint32_t b = __builtin_amdgcn_readlane(beg, k), e = __builtin_amdgcn_readlane(end, k);
            if (b >= lim) return;                                                // past the chunk (or past the last tensor: b = n)
            // (readlane returns int: through uint32_t, or the low word's bit 31 would smear over the high word)
            const uintptr_t p = (uintptr_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)ptr, k) |
                                ((uintptr_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(ptr >> 32), k) << 32);
            body(b, e, p);
        }
        s0 += 64u;
    }
}

__device__ __forceinline__ void load_seg(const GroupView &g, const Chunk &c, float (&v)[kSteps])
{
    const uintptr_t entry = chunk_entry(g, c);
    if (!(entry & 1u)) {
        const float *p = reinterpret_cast<const float *>(entry) + c.lane;
#pragma unroll
        for (int j = 0; j < kSteps; ++j) v[j] = ld_stream(p + 64 * j);
    } else {
#pragma unroll
        for (int j = 0; j < kSteps; ++j) v[j] = 0.0f;
        for_each_tensor_of_chunk(g, c, (uint32_t)(entry >> 1), [&](uint32_t beg, uint32_t end, uintptr_t ptr) {
            const float *p = reinterpret_cast<const float *>(ptr);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                const uint32_t i = c.base + 64 * j + c.lane;
                if (i >= beg && i < end) v[j] = p[i - beg];
            }
        });
    }
}

// (Measured on this part: stores whose 256-byte wave windows miss a 64-byte boundary are slower -- a bare
// 102 MB fill takes 16 us aligned and 22 us not, the plane decompress kernel 27 and 32 us -- while loads
// are not sensitive.  Rotating lanes to aligned windows did not pay in these kernels.  Tensors whose flat
// offset is a multiple of 16 elements keep the aligned rate.)
__device__ __forceinline__ void store_seg(const GroupView &g, const Chunk &c, const float (&v)[kSteps], uintptr_t entry)
{
    if (!(entry & 1u)) {
        float *p = reinterpret_cast<float *>(entry) + c.lane;
#pragma unroll
        for (int j = 0; j < kSteps; ++j) st_stream(p + 64 * j, v[j]);
    } else {
        for_each_tensor_of_chunk(g, c, (uint32_t)(entry >> 1), [&](uint32_t beg, uint32_t end, uintptr_t ptr) {
            float *p = reinterpret_cast<float *>(ptr);
#pragma unroll
            for (int j = 0; j < kSteps; ++j) {
                const uint32_t i = c.base + 64 * j + c.lane;
                if (i >= beg && i < end) p[i - beg] = v[j];
            }
        });
    }
}
__device__ __forceinline__ void store_seg(const GroupView &g, const Chunk &c, const float (&v)[kSteps])
{
    store_seg(g, c, v, chunk_entry(g, c));
}
// v in the rotated mapping, rot = chunk_rotation(entry) (0 when the chunk has no address of its own)
__device__ __forceinline__ void store_seg_rot(const GroupView &g, const Chunk &c, const float (&v)[kSteps], uintptr_t entry, uint32_t rot)
{
    if (!(entry & 1u)) {
        // steps 0..14 at constant offsets from one address (they fold into the instructions), step 15 may wrap
        float *p = reinterpret_cast<float *>(entry), *q = p + (c.lane + rot);
#pragma unroll
        for (int j = 0; j < kSteps - 1; ++j) st_stream(q + 64 * j, v[j]);
        st_stream(p + rotated(kSteps - 1, c.lane, rot), v[kSteps - 1]);
    } else {
        store_seg(g, c, v, entry);
    }
}

// ---- packed bit planes -------------------------------------------------------
// Store the 16 ballots of a chunk (32 words) to a plane of `nwords` words.
// `stage` is 16 uint64 of LDS private to the calling wavefront.
__device__ __forceinline__ void store_plane(uint32_t *plane, uint32_t nwords, const Chunk &c,
                                            const uint64_t (&ballots)[kSteps], uint64_t *stage)
{
#pragma unroll
    for (int j = 0; j < kSteps; ++j) if (c.lane == (uint32_t)j) stage[j] = ballots[j];
    __builtin_amdgcn_wave_barrier();
    if (c.lane < 32) {
        uint32_t w = (c.base >> 5) + c.lane;
        if (w < nwords) plane[w] = reinterpret_cast<const uint32_t *>(stage)[c.lane];
    }
    __builtin_amdgcn_wave_barrier();
}

// ---- reductions ----------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}
__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
    return x;
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves inside the vector ALU (three shifts by one,
// two and three lanes, shifts by four and eight inside the rows of 16, then the row totals handed on: seven adds) instead
// of six rounds through the LDS crossbar that a shuffle-based scan takes: about 30 against 600 cycles of latency, which
// counts in kernels that do little else than wait.  All 64 lanes must be active.
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t x)
{
    uint32_t v = x;
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);      // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);      // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x113, 0xf, 0xf, true);      // row_shr:3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xe, true);      // row_shr:4, lanes 4..15 of a row
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xc, true);      // row_shr:8, lanes 8..15
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, true);      // row_bcast:15 into rows 1 and 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, true);      // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ uint32_t wave_total(uint32_t incl) { return (uint32_t)__builtin_amdgcn_readlane((int)incl, 63); }

// all threads of the block get the block total; fixed combination order
__device__ __forceinline__ double block_sum(double x, double *lds4)
{
    x = wave_sum(x);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = x;
    __syncthreads();
    double t = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
    __syncthreads();
    return t;
}
__device__ __forceinline__ float block_max(float x, float *lds4)
{
    x = wave_max(x);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = x;
    __syncthreads();
    float t = fmaxf(fmaxf(lds4[0], lds4[1]), fmaxf(lds4[2], lds4[3]));
    __syncthreads();
    return t;
}

// number of set bits of a ballot below this lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

// ---- Philox-4x32-10 (Salmon et al., SC'11) --------------------------------------
// Counter = (J lo, J hi, worker, iteration), J = global element index / 4, key =
// seed; the element takes output word (index % 4), top 24 bits scaled to [0, 1).
// a ^ b ^ k in one instruction (the three-input bit operation with the truth table of xor); k is the same for the
// whole wavefront (a round key: it lives in a scalar register).  The compiler emits two two-input operations for
// the same expression, and where the quantizers' pass over p is bound by the vector ALU that shows: QSGD compress
// 84.2 -> 82.4 us.
__device__ __forceinline__ uint32_t xor3_uniform(uint32_t a, uint32_t b, uint32_t k)
{
    uint32_t r;
    asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x96" : "=v"(r) : "v"(a), "v"(b), "s"(k));
    return r;
}

__device__ __forceinline__ void philox4x32_10(uint64_t seed, uint32_t worker, uint32_t iter_lo, uint64_t J, uint32_t (&out)[4])
{
    uint32_t c0 = (uint32_t)J, c1 = (uint32_t)(J >> 32), c2 = worker, c3 = iter_lo;
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32 x 32 -> 64 multiply each (two instructions instead of four on the quarter-rate multiplier)
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0, hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        c0 = xor3_uniform(hi1, c1, k0);
        c1 = lo1;
        c2 = xor3_uniform(hi0, c3, k1);
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ float u01(uint32_t x) { return (float)(x >> 8) * 5.9604644775390625e-8f; }

template <int R>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t x)      // value of lane R of each group of four lanes
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, R | (R << 2) | (R << 4) | (R << 6), 0xF, 0xF, true);
}

// The Philox words of a chunk's 16 steps for this lane (element gbase + 64 j + lane in step j
// takes word (index % 4) of block index / 4).
// Four adjacent lanes hold four consecutive elements; when gbase is a multiple of 4 these
// share one Philox block, so each lane computes one block per four steps (the one of step
// 4m + lane % 4) and the four words are handed round inside the quad.
__device__ __forceinline__ void chunk_words(uint64_t seed, uint32_t worker, uint32_t iter_lo, uint64_t gbase, uint32_t lane,
                                            uint32_t (&x)[kSteps])
{
    if ((gbase & 3u) == 0) {
        const uint32_t me = lane & 3u;
#pragma unroll
        for (int m = 0; m < kSteps / 4; ++m) {
            uint32_t w[4];
            philox4x32_10(seed, worker, iter_lo, (gbase + 64u * (4 * m + me) + lane) >> 2, w);
            uint32_t y[4][4];                      // y[r][i]: word i of the block of step 4m + r
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                y[0][i] = quad_bcast<0>(w[i]); y[1][i] = quad_bcast<1>(w[i]);
                y[2][i] = quad_bcast<2>(w[i]); y[3][i] = quad_bcast<3>(w[i]);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
                x[4 * m + r] = me == 0 ? y[r][0] : me == 1 ? y[r][1] : me == 2 ? y[r][2] : y[r][3];
        }
    } else {
        // The chunk starts s = gbase % 4 elements into a Philox block (a group whose tensors before it do not add up to
        // a multiple of 4).  With v = lane + s, the element of step j sits in block B0 + 16 j + v / 4, word v % 4: the
        // same 256 blocks as above, B0 + 16 j + q computed by lane 4 q + j % 4, plus one more, B0 + 256, that only the
        // last s lanes need in step 15 (every lane computes it: five blocks per lane instead of the sixteen of a block
        // per element).  A lane with v >= 64 is served by quad 0's blocks of the next step.  The lanes that share a
        // block are no aligned quad any more, so the words travel through ds_bpermute.
        // (Measured, compress of such a group of 25.6 M elements: QSGD 118.5 -> 86.8 us, TernGrad 105.9 -> 86.0, Rand-k 94.8 -> 86.7:
        // what a group that starts on a block takes.)
        const uint32_t s = (uint32_t)gbase & 3u, v = lane + s, i = v & 3u;
        const uint64_t B0 = (gbase - s) >> 2;
        const uint32_t me = lane & 3u, quad = lane >> 2;
        const bool over = v >= 64u;
        uint32_t w[kSteps / 4][4], wl[4];
#pragma unroll
        for (int m = 0; m < kSteps / 4; ++m) philox4x32_10(seed, worker, iter_lo, B0 + 16u * (4 * m + me) + quad, w[m]);
        philox4x32_10(seed, worker, iter_lo, B0 + 256u, wl);
#pragma unroll
        for (int j = 0; j < kSteps; ++j) {
            const int m = j >> 2, r = j & 3;
            const uint32_t src = over ? (uint32_t)((j + 1) & 3) : ((v >> 2) << 2) + (uint32_t)r;     // the lane that computed the block
            uint32_t got[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) got[t] = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(src << 2), (int)w[m][t]);
            uint32_t val = i == 0 ? got[0] : i == 1 ? got[1] : i == 2 ? got[2] : got[3];
            if (r == 3) {            // for the lanes with v >= 64 the next step's block comes out of the next round of four
                uint32_t alt[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    alt[t] = j + 1 < kSteps ? (uint32_t)__builtin_amdgcn_ds_bpermute((int)(src << 2), (int)w[(m + 1) & 3][t]) : wl[t];
                const uint32_t a = i == 0 ? alt[0] : i == 1 ? alt[1] : i == 2 ? alt[2] : alt[3];
                val = over ? a : val;
            }
            x[j] = val;
        }
    }
}

// the same as uniforms in [0, 1)
__device__ __forceinline__ void chunk_uniforms(uint64_t seed, uint32_t worker, uint32_t iter_lo, uint64_t gbase, uint32_t lane,
                                               float (&u)[kSteps])
{
    uint32_t x[kSteps];
    chunk_words(seed, worker, iter_lo, gbase, lane, x);
#pragma unroll
    for (int j = 0; j < kSteps; ++j) u[j] = u01(x[j]);
}

}  // namespace mc
