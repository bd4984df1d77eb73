// Host <-> kernel-launcher interface of the library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/mergecomp.h"
#include "mc_device.h"

namespace mc {

constexpr uint32_t kMagic = 0x3150434Du;
constexpr int kHeaderBytes = 128;     // bodies of payload and state start on a 128-byte cache line
constexpr int kMaxWorkers = 64;

struct PayloadHeader {          // one cache line, see the layout in mergecomp.h
    uint32_t magic, algo;
    uint64_t n, k;
    float scale;
    uint32_t levels;
    uint32_t pad[24];           // pad[0]: OneBit's mean of the negative class; the rest zero
};
static_assert(sizeof(PayloadHeader) == kHeaderBytes, "payload header is one 128-byte line");

struct StateHeader {            // one cache line in front of the error-feedback floats
    float scale;                // EF-Sign: scale of the last call; OneBit: mean of its upper class (0 after zero-fill / import)
    float scale_lo;             // OneBit: mean of the lower class of the last call
    uint32_t prev_worker, prev_iter;   // QSGD / TernGrad: whose random stream the last call drew from (scale: its norm / max)
    uint32_t sent_key;          // Top-k, DGC: elements of the last call whose key exceeds this were sent and count as 0 (see sparse_accum_k)
    uint32_t pad[27];
};
static_assert(sizeof(StateHeader) == kHeaderBytes, "state header is one 128-byte line");

// DGC keeps two vectors in the state: v[n] first, then u[n] from the next multiple of 32 floats on, so that both start
// on a 128-byte line (a chunk's stores then cover whole lines).
__host__ __device__ inline size_t dgc_u_offset(uint32_t n) { return ((size_t)n + 31u) & ~(size_t)31u; }

struct PayloadPtrs { const uint8_t *p[kMaxWorkers]; };
struct PtrChunk { uintptr_t p[256]; };

// radix-select state carried between the passes of the exact top-k
struct SelectState {
    uint32_t lo;         // the threshold key lies in [lo, lo + range of the levels still to resolve)
    uint32_t mode;       // what the seed kernel found (fast / refill flags)
    uint64_t need;       // entries still to take among the keys of that range
};

// profiling slots
enum KernelId {
    K_UPLOAD = 0, K_EFSIGN_COMPRESS, K_SCALAR_FINALIZE, K_ACCUM_REDUCE, K_QSGD_ENCODE, K_TERN_ENCODE,
    K_FP16_COMPRESS, K_DENSE_DECOMPRESS, K_SPARSE_ACCUM, K_SPARSE_SEED, K_CAND_HIST2, K_CAND_HIST3, K_CAND_COUNT,
    K_CAND_EMIT, K_SPARSE_DECOMPRESS, K_STATE_CONVERT, K_LEAN_SELECT, K_LEAN_EMIT, K_SPARSE_SLOW, K_COUNT
};

// reduction kinds of the two-pass quantizers
enum ReduceMode { RED_MEAN_ABS = 0, RED_L2 = 1, RED_MAX_ABS = 2, RED_ONE = 3, RED_MEANS = 4 };
// the one-bit compressors (one kernel) and what their single plane decodes to
enum SignMode { SIGN_EF = 0, SIGN_MEANS = 1, SIGN_PLAIN = 2, SIGN_MOMENTUM = 3 };
enum PlaneKind { PLANE_SCALE = 0, PLANE_MEANS = 1, PLANE_VOTE = 2 };

struct LaunchCtx {               // what a launcher needs besides its arguments
    hipStream_t stream;
    void *prof;                  // opaque: profiling recorder or null
    mutable hipEvent_t ev_a = nullptr, ev_b = nullptr;   // set by prof_begin when the next launch is to be timed
};
// prof_begin arms the next MC_LAUNCH with a start / stop event pair (if that kernel slot is being timed);
// the events are attached to the dispatch itself, so they bracket the kernel's execution only.
void prof_begin(const LaunchCtx &lc, int id);
void prof_end(const LaunchCtx &lc, int id);
#define MC_LAUNCH(kernel, grid, block, lc, ...)                                                                       \
    do {                                                                                                              \
        if ((lc).ev_a) hipExtLaunchKernelGGL(kernel, grid, block, 0, (lc).stream, (lc).ev_a, (lc).ev_b, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel, grid, block, 0, (lc).stream, __VA_ARGS__);                                    \
    } while (0)

// ---- dense kernels (kernels_dense.hip) -----------------------------------------
void launch_upload_ptrs(const LaunchCtx &lc, const uintptr_t *host, uintptr_t *dev, uint32_t count);
void launch_expand_ptrs(const LaunchCtx &lc, const GroupView &g, uintptr_t *chunk_addr);
void launch_sign_compress(const LaunchCtx &lc, int mode, const GroupView &g, bool ef, float *state_f, const StateHeader *prev,
                          float beta, uint32_t *words, uint32_t nwords, double *partial, PayloadHeader *hdr, uint32_t algo);
void launch_scalar_finalize(const LaunchCtx &lc, const double *partial, uint32_t nblocks, int mode, uint32_t n,
                            PayloadHeader *hdr, uint32_t algo, uint64_t k, uint32_t levels, float *state_scale);
void launch_accum_reduce(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, const StateHeader *prev, int mode,
                         uint32_t levels, uint64_t seed, double *partial);
void launch_qsgd_encode(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, StateHeader *sh, const PayloadHeader *hdr,
                        int8_t *codes, uint32_t levels, uint64_t seed, uint32_t worker, uint32_t iter_lo);
void launch_tern_encode(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, StateHeader *sh, const PayloadHeader *hdr,
                        uint32_t *planes, uint32_t nwords, uint64_t seed, uint32_t worker, uint32_t iter_lo);
void launch_fp16_compress(const LaunchCtx &lc, const GroupView &g, bool ef, float *state_f, PayloadHeader *hdr,
                          uint16_t *halves);
void launch_dense_decompress(const LaunchCtx &lc, int algo, const GroupView &out, const PayloadPtrs &pl, int W,
                             float alpha, uint32_t levels, int *status);
void launch_state_convert(const LaunchCtx &lc, int algo, bool to_residual, uint32_t n, const void *src, void *dst, uint32_t levels,
                          uint64_t seed, uint64_t goff);

// ---- sparse kernels (kernels_sparse.hip) ----------------------------------------
constexpr int kHintWorkers = 64;                         // hints kept per group, one per worker id modulo this
constexpr int kHintWords = 4;                            // words of a hint record (filter key, halvings of the margin, calls it is held after a miss, cap on the halvings)
constexpr int kWinCopies = 8;                                // copies of the window histogram (a block adds to the copy of its index)
constexpr int kHistWords = 2048 * kWinCopies + 2048 + 1024 + 2048 + 64;   // bins of the window and of the three radix levels, copies of the window's open bin

// The keys that share the threshold's window bin (the only candidates whose fate the window does not settle) are
// handed from the select kernel to the emit kernel as an unordered list, appended to by wave-wide atomic adds.
// Adds to one address queue up behind each other, so the list is kept in kUSub sublists (a wavefront appends to the
// one of its tile index) whose counters sit on cache lines of their own.
constexpr int kUSub = 64;
constexpr uint32_t kUCap = 4096;      // keys in the threshold's window bin that the two-kernel route takes; a sublist holds as many
constexpr int kUCountStride = 32;     // words between sublist counters (one 128-byte line each)
struct UEntry { uint32_t idx, bits; };       // group-relative index, candidate bits

struct SparseScratch {
    uint32_t *hist;        // kHistWords counters; each level is cleared by a later kernel of the same call
    SelectState *sel;      // [0]: after the seed, [1..3]: after each radix level
    uint32_t *hint;        // this (group, worker)'s hint record; word 0: keys >= it are candidates (0 = everything)
    uint32_t *cand_bits;   // candidate values (fp32 bit patterns), 1024 slots per chunk, filled from the front
    uint16_t *cand_loc;    // candidate positions inside their chunk
    uint64_t *tile_runs;   // candidates of the four chunks of every tile, 16 bits each
    uint32_t *tile_cnt;    // per tile: candidates above (low 16 bits) / equal to (high 16 bits) the threshold
    uint32_t *blk_cnt;     // the same per block of four tiles
    UEntry *ulist;         // kUSub sublists of kUCap entries: the candidates in the threshold's window bin
    uint32_t *ucount;      // their lengths, kUCountStride words apart; cleared by the streaming pass of the next call
    uint32_t *sync;        // [0]: arrivals at the grid-wide barriers of the slow routes (cleared by the streaming pass); [32..36): calls per route
    uint32_t spin_limit;   // polls after which a block gives up waiting at such a barrier (mc_set_barrier_spin_limit)
};
// sync_blocks: how many blocks of 1024 threads the device surely holds at once (one per compute unit): the slow routes
// of the selection run on that many blocks with grid-wide barriers between their steps
void launch_sparse_compress(const LaunchCtx &lc, int algo, const GroupView &g, bool ef, float *state_f, float momentum,
                            uint64_t k, PayloadHeader *hdr, const SparseScratch &sc, uint64_t seed, uint32_t worker, uint32_t iter_lo,
                            uint32_t sample_stride, uint32_t sample_first, uint64_t sample_need, uint32_t sync_blocks, int *status);
void launch_sparse_decompress(const LaunchCtx &lc, int algo, const GroupView &out, const PayloadPtrs &pl, int W,
                              float alpha, uint64_t k, int *status, bool capped);

}  // namespace mc
