/*
 * mergecomp.h -- C ABI of the MI355X (gfx950) MergeComp hot path.
 *
 * The library implements the two per-group steps of the paper's Algorithm 1,
 *     delta = C(g)                      -> mc_compress
 *     g~    = aggregate(C^-1(Delta))    -> mc_decompress_sum
 * for a model whose N gradient tensors have been partitioned into y contiguous
 * groups (Section 4.1: tensors of a group are merged and compressed together in
 * one compression operation; Section 4.3: a partition X_y = {x_1..x_y}), plus
 * the partition helper itself (mc_partition).
 *
 * Conventions
 *   - "host" / "device" is stated for every pointer.  The library never takes
 *     ownership of a caller buffer.  It owns only the context (small device
 *     tables and scratch allocated in mc_ctx_create, freed in mc_ctx_destroy).
 *   - mc_compress / mc_decompress_sum only enqueue kernels on the caller's HIP
 *     stream (void* = hipStream_t, NULL = the default stream).  They allocate
 *     nothing on the device or the host (the optional per-kernel profiler
 *     creates HIP events while it is enabled), never synchronise the host with
 *     the device and read nothing back.  All calls that use one context must be issued in stream order
 *     (one stream, or streams the caller has ordered with events): the context
 *     scratch and its cached pointer tables are shared between calls.
 *     The calls are not meant to be recorded into a HIP graph: iteration and
 *     worker numbers and the tensor addresses travel as kernel arguments, so a
 *     replay would repeat the random stream of the recorded call.
 *   - A group is addressed as the flat fp32 vector obtained by concatenating
 *     its tensors in list order, each tensor contiguous; nothing is copied to
 *     build it, kernels walk a segment table.  Flat index i of group j has the
 *     model-global index  (elements of groups 0..j-1) + i.
 *   - fp32 element arithmetic is IEEE binary32, round-to-nearest-even, without
 *     fused multiply-add; group reductions are accumulated in fp64.
 *   - Return value: 0 on success, a negative mc_status otherwise.  No call
 *     throws or aborts.  Non-finite gradient values give unspecified codes.
 *
 * Payload layout (little endian), identical for every algorithm up to the body:
 *   byte  0  uint32  magic 0x3150434D
 *   byte  4  uint32  algorithm id (mc_algo)
 *   byte  8  uint64  n, elements of the group
 *   byte 16  uint64  k, kept entries (sparsifiers; 0 otherwise)
 *   byte 24  float   group scalar: EF-Sign scale, QSGD norm, TernGrad max, OneBit mean of the
 *                    non-negative class, SignSGD / SigNUM 1.0 (0 otherwise)
 *   byte 28  uint32  QSGD levels s; DGC with a sampled threshold: capacity c of the entry arrays (0 otherwise)
 *   byte 32  float   OneBit mean of the negative class (0 otherwise)
 *   byte 36..127     zero (the header fills one 128-byte cache line, so that the body starts on a line)
 *   byte 128 body:
 *     EF-Sign, OneBit, SignSGD, SigNUM
 *               ceil(n/32) uint32; element i <-> bit (i%32) of word i/32, 1 = non-negative; pad bits 0
 *     TernGrad  non-zero plane ceil(n/32) uint32, then negative plane, same bit order
 *     QSGD      n int8 codes in [-s, s], zero-padded to a multiple of 4 bytes
 *     FP16      n binary16, zero-padded to a multiple of 4 bytes
 *     Top-k, DGC, Rand-k
 *               idx[k] uint32 ascending group-relative indices, then val[k] float, then the directory of the
 *               index list, dir[ceil(n/4096) + 1] uint32: dir[t] = number of entries with index below 4096 t
 *               (dir[0] = 0, the last entry = k; no directory when n = 0).  It repeats what the index list says,
 *               so that a receiver finds a payload's share of a 4096-element span without a search; a
 *               directory that disagrees with its list makes the sums unspecified, never an access out of bounds
 *               (DGC with a sampled threshold: idx[c] then val[c], the first k of each in use, the rest zero,
 *               then the directory)
 *   Payload buffers must be 16-byte aligned; 128-byte alignment is what the kernels are fastest with
 *   (measured: FP16 decompress-sum of 8 payloads 81 us against 95 us with bodies 64 bytes off the lines).
 */
#ifndef MERGECOMP_H
#define MERGECOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mc_ctx mc_ctx;

/* Compression algorithms (Section 2.1 and Table 1 name them; the paper gives no
 * formulas, the definitions of the cited original works are used). */
typedef enum {
    MC_ALGO_EFSIGN = 1,   /* 1-bit sign with per-group scale mean|p| and error feedback       */
    MC_ALGO_TOPK = 2,     /* exact top-k of |p|, ties broken towards the lower index          */
    MC_ALGO_DGC = 3,      /* momentum correction + exact top-k + momentum factor masking      */
    MC_ALGO_QSGD = 4,     /* stochastic rounding to s levels of |p|/||p||_2 (Section 5: 8 bit) */
    MC_ALGO_TERNGRAD = 5, /* ternary {-s,0,+s}, s = max|p|, Bernoulli(|p|/s)                   */
    MC_ALGO_FP16 = 6,     /* binary16 cast, round to nearest even                              */
    /* the other four schemes of Table 1 */
    MC_ALGO_SIGNSGD = 7,  /* sign(g), no memory; aggregated by majority vote: sign of the sum   */
    MC_ALGO_SIGNUM = 8,   /* sign of the momentum m = beta m + (1-beta) g; majority vote         */
    MC_ALGO_ONEBIT = 9,   /* 1 bit, decoded as the mean of its class (p>=0 / p<0); error feedback */
    MC_ALGO_RANDK = 10    /* k positions drawn uniformly (largest Philox keys); error feedback   */
} mc_algo;

/* Partition policies for mc_partition. */
typedef enum {
    MC_PART_EVEN_COUNT = 0, /* the "naive" strategy of Section 5.2: even by number of tensors   */
    MC_PART_EVEN_ELEMS = 1, /* even by number of elements                                        */
    MC_PART_USER = 2        /* caller-supplied boundaries (what Algorithm 2 would return)        */
} mc_part_policy;

typedef enum {
    MC_OK = 0,
    MC_ERR_INVALID_ARG = -1, /* null pointer, unknown algo/policy, bad config value             */
    MC_ERR_RANGE = -2,       /* y > N, group with >= 2^32 - 2^24 elements, bounds not increasing */
    MC_ERR_ALLOC = -3,       /* host or device allocation failed in mc_ctx_create                */
    MC_ERR_DEVICE = -4,      /* a HIP runtime call failed, or (mc_last_device_status) a bounded wait inside
                                a kernel of the sparsifiers' rare selection routes ran out               */
    MC_ERR_PAYLOAD = -5      /* a payload header did not match the context (device-side check)   */
} mc_status;

typedef struct {
    int32_t algo;        /* mc_algo                                                             */
    int32_t use_ef;      /* 1: p = g + e and the residual e is updated; 0: p = g, state unused.
                            Must be 1 for DGC, SigNUM, Rand-k (they always carry state), 0 for SignSGD */
    uint32_t ratio_ppm;  /* sparsifiers: kept fraction in parts per million (Section 5: 10000)   */
    int32_t qsgd_bits;   /* QSGD code width incl. sign, 2..8; levels s = 2^(bits-1) - 1          */
    float dgc_momentum;  /* DGC momentum m; SigNUM beta                                          */
    uint32_t dgc_sample_ppm; /* DGC only (else 0): 0 = exact top-k.  Otherwise the threshold is the one that keeps
                            ratio_ppm of a SAMPLE of this rate (every floor(1e6/rate)-th element from a Philox-drawn
                            start), everything reaching it is sent, and the payload has room for 2k entries   */
    uint64_t seed;       /* Philox key of the stochastic quantizers and of Rand-k                */
} mc_config;

/*
 * Partition a list of N tensors into y contiguous groups (Section 4.3; Lemma 1
 * counts exactly these partitions).  Host-only, touches no device.
 *   numel        host, N tensor sizes in elements (>= 0)
 *   user_bounds  host, y+1 boundaries for MC_PART_USER, otherwise ignored (may be NULL)
 *   bounds_out   host, y+1 entries: 0 = b[0] < b[1] < ... < b[y] = N; group j = tensors [b[j], b[j+1])
 * Errors: MC_ERR_INVALID_ARG (null, N < 1, y < 1, negative size, unknown policy),
 *         MC_ERR_RANGE (y > N, user bounds not strictly increasing from 0 to N).
 */
int mc_partition(const int64_t *numel, int32_t n_tensors, int32_t y, int32_t policy,
                 const int32_t *user_bounds, int32_t *bounds_out);

/*
 * Iteration-time model of Section 4.3 and the partition search of Algorithm 2.  Host-only.
 *
 * F(X_y) = A + sum h(x_i) + sum g(x_i) - sum p(x_i) with the linear overheads of Assumption 5 (Section 4.3),
 * h(x) = B_h + gamma_h x (compression) and g(x) = B_g + gamma_g x (communication), x in elements.
 * The overlap p is not given in closed form by the paper; the schedule it describes (wait-free
 * back-propagation, proof of Theorem 3) is evaluated directly: the GPU runs the forward pass
 * (fwd_time), then back-propagation tensor by tensor in list order (bwd_time[t] seconds each) and
 * compresses a group as soon as its last tensor is done; the network sends group i when it has been
 * compressed and group i-1 has been sent.  F is the time at which the last group has been sent.
 */
typedef struct {
    double fwd_time;  /* seconds of the iteration before back-propagation starts            */
    double B_h;       /* compression: seconds per group (the B_h of Lemma 2)                */
    double gamma_h;   /* compression: seconds per element                                   */
    double B_g;       /* communication: seconds per group                                   */
    double gamma_g;   /* communication: seconds per element                                 */
} mc_time_model;

/* F of the partition `bounds` (y+1 entries as returned by mc_partition).  All pointers host.
 * Errors: MC_ERR_INVALID_ARG (null, N < 1, y < 1), MC_ERR_RANGE (y > N, bounds not increasing 0..N). */
int mc_partition_cost(const int64_t *numel, const double *bwd_time, int32_t n_tensors, const mc_time_model *model,
                      const int32_t *bounds, int32_t y, double *F_out);

/*
 * Algorithm 2: for y = 2 .. Y find X_y* = argmin F over all partitions into y contiguous groups
 * and stop at y-1 if F_min(y-1) < F_min(y), at y if F_min(y-1) - F_min(y) < alpha F_min(y-1).
 * The inner argmin is exact: F is monotone in the time the network becomes free, so a dynamic
 * programme over (last tensor, groups used) finds it in O(N^2 y) instead of the O(N^(y-2) log N)
 * enumeration of Theorem 3.
 *   bounds_out  host, at least min(Y, N) + 1 entries; receives y_out + 1 boundaries
 *   y_out       host, number of groups of the partition returned
 *   F_out       host, its F (may be NULL)
 * Errors: MC_ERR_INVALID_ARG (null, N < 1, Y < 1, alpha outside [0, 1), negative time), MC_ERR_ALLOC.
 */
int mc_partition_search(const int64_t *numel, const double *bwd_time, int32_t n_tensors, const mc_time_model *model,
                        int32_t Y, double alpha, int32_t *bounds_out, int32_t *y_out, double *F_out);

/*
 * Create a context for one (config, tensor list, partition) on the current HIP
 * device.  All arrays are host memory and are copied.  Allocates the device
 * segment tables and scratch for every group, and reserves the host-side lists the
 * hot calls fill, so that those allocate nothing.
 * Device memory held by a context, with T = tiles of 4096 elements of its largest group:
 *   every algorithm   24 T bytes of reduction partials; up to 256 cached tensor-address lists with one
 *                     8-byte address per 1024 elements each (32 T bytes per list, 256 MiB at most in all)
 *   sparsifiers       6 bytes per element of the largest group for candidate values and positions
 *                     (24576 T; 153 MB for a 25.6 M element group), 12.25 T bytes of per-tile counts, 2 MiB for the
 *                     list of keys in the threshold's histogram bin, histograms and counters of about 100 KB
 */
int mc_ctx_create(mc_ctx **out, const mc_config *cfg, const int64_t *numel, int32_t n_tensors,
                  const int32_t *bounds, int32_t y);
int mc_ctx_destroy(mc_ctx *ctx);

/* Elements n of a group / entries of a sparsifier's payload (0 for other algorithms) / number of
 * tensors of the group.  mc_group_k is the exact kept count k = min(n, max(1, floor(n*ppm/1e6))); for DGC
 * with a sampled threshold (dgc_sample_ppm != 0) it is the payload's capacity min(n, 2k), of which the
 * header of each payload says how many entries are in use. */
int64_t mc_group_numel(const mc_ctx *ctx, int32_t group);
int64_t mc_group_k(const mc_ctx *ctx, int32_t group);
int32_t mc_group_tensors(const mc_ctx *ctx, int32_t group);

/* Exact size of a group's payload (static: k is exact, so no size read-back) and
 * of its error-feedback memory.  0 for an invalid group. */
size_t mc_payload_bytes(const mc_ctx *ctx, int32_t group);
size_t mc_state_bytes(const mc_ctx *ctx, int32_t group);

/*
 * delta = C(g) for one group of one worker (Algorithm 1), fused with the
 * error-feedback update (Section 3.2: error feedback costs another decode).
 *   worker, iter  select the random stream of QSGD / TernGrad / Rand-k / the sampled DGC (counter words: worker, and
 *                 the low 32 bits of iter: streams repeat after 2^32 iterations); a sparsifier also keeps its
 *                 candidate-filter hint per (group, worker modulo 64)
 *   grad_ptrs     host array, one DEVICE pointer per tensor of the group (fp32, contiguous,
 *                 4-byte aligned; 16-byte alignment enables the fastest path); read only
 *   state         device, mc_state_bytes() bytes, 16-byte aligned (128-byte alignment is fastest: the
 *                 floats then start on a cache line), zero-filled by the caller
 *                 before the first iteration and otherwise opaque: a 128-byte header followed by
 *                 n floats (DGC: v[n], then u[n] from the next multiple of 32 floats on).  For EF-Sign,
 *                 OneBit, QSGD and TernGrad the floats hold p = g + e of the last call and the header
 *                 its group scalars (QSGD, TernGrad: also whose random stream it drew from), from which
 *                 the residual is re-derived; use mc_state_export_residual to read e.
 *                 May be NULL when use_ef = 0.
 *   payload_out   device, mc_payload_bytes() bytes, 16-byte aligned; fully overwritten
 */
int mc_compress(mc_ctx *ctx, int32_t group, uint32_t worker, uint64_t iter,
                const float *const *grad_ptrs, void *state, void *payload_out, void *stream);

/*
 * mc_compress for callers that cannot allocate device memory and must not have it allocated on their behalf
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments, same
 * payload and state, bit for bit; the difference is where the kernels keep their per-tile reduction partials:
 * not in the context's scratch but in a device array of fixed size that is part of the library's code object
 * (mc_static_scratch_bytes() = 384 KiB, held by every GPU the library runs on until the process ends).  Calls
 * neither hipMalloc nor hipFree nor any allocating routine, and records no profiler events.
 *   Limits   a group of at most mc_static_max_elems() = 2^26 elements (MC_ERR_RANGE above);
 *            EF-Sign, OneBit, SignSGD, SigNUM, QSGD, TernGrad, FP16 only: the sparsifiers return
 *            MC_ERR_INVALID_ARG (their candidate scratch grows with 6 bytes per element and stays in
 *            the context)
 *   Sharing  all calls on one GPU, from every context, use the same array: calls that may overlap on one
 *            GPU (different streams without ordering, several host threads) race on it and must be ordered
 *            by the caller.  Nothing in it has to start at zero: every call overwrites what it reads.
 */
int mc_compress_static(mc_ctx *ctx, int32_t group, uint32_t worker, uint64_t iter,
                       const float *const *grad_ptrs, void *state, void *payload_out, void *stream);
size_t mc_static_scratch_bytes(void);
int64_t mc_static_max_elems(void);

/*
 * g~ = aggregate(C^-1(Delta)) for one group (Algorithm 1): decode the W workers'
 * payloads and write  out_i = alpha * (((0 + d_0,i) + d_1,i) + ... + d_{W-1,i})  in fp32.
 *   payloads   host array of W DEVICE pointers to payloads of this group, 1 <= W <= 64 (MC_ERR_RANGE above)
 *   out_ptrs   host array, one DEVICE pointer per tensor of the group; fully overwritten
 * A payload whose header does not match (magic, algorithm, n, k) is reported through
 * mc_last_device_status; out-of-range sparse indices are ignored, never written.
 */
int mc_decompress_sum(mc_ctx *ctx, int32_t group, const void *const *payloads, int32_t W, float alpha,
                      float *const *out_ptrs, void *stream);

/*
 * The loops of Algorithm 1 over all groups of the context in one call each, in group order, for a caller whose
 * gradients are all there already (no overlap with back-propagation) -- the same kernels as y calls of
 * mc_compress / mc_decompress_sum, without y trips through the caller's language binding.
 *   grad_ptrs_all  host array, one DEVICE pointer per tensor of the MODEL (the list given to mc_ctx_create)
 *   states         host array of y DEVICE pointers, states[j] as `state` of mc_compress for group j (NULL when use_ef = 0)
 *   payloads_out   host array of y DEVICE pointers, payloads_out[j] receives group j's payload
 *   payloads       host array of W * y DEVICE pointers: payloads[w * y + j] is worker w's payload of group j
 *   out_ptrs_all   host array, one DEVICE pointer per tensor of the model
 * Stops at the first group that returns an error and returns it.
 */
int mc_compress_groups(mc_ctx *ctx, uint32_t worker, uint64_t iter, const float *const *grad_ptrs_all, void *const *states,
                       void *const *payloads_out, void *stream);
int mc_decompress_sum_groups(mc_ctx *ctx, const void *const *payloads, int32_t W, float alpha, float *const *out_ptrs_all,
                             void *stream);

/*
 * Convert between the opaque state and plain error-feedback memory
 * (n floats e; DGC: v[n] then u[n]), both DEVICE pointers.  Import of a residual
 * followed by export returns the same bits.
 */
int mc_state_export_residual(mc_ctx *ctx, int32_t group, const void *state, float *e_out, void *stream);
int mc_state_import_residual(mc_ctx *ctx, int32_t group, const float *e_in, void *state, void *stream);

/* Synchronises the context's device and returns MC_OK, MC_ERR_PAYLOAD if any
 * mc_decompress_sum since the last call saw a mismatching header, or MC_ERR_DEVICE if a
 * sparsifier's mc_compress gave up waiting at a grid-wide barrier of its rare selection routes
 * (the blocks of that kernel wait for each other, at most about two seconds, which needs them all
 * resident: other work that holds the GPU's compute units for that long can cause it; the
 * payload of that call is then incomplete and its error-feedback state unspecified -- import a
 * residual again before the next call; the context itself stays usable).  Clears the flag. */
int mc_last_device_status(mc_ctx *ctx);

/* For tests of the error path above: how often a block looks at a grid-wide barrier before it gives up
 * (0 = the default, 2^21 looks of about a microsecond; 1 = after the first look, which makes every
 * mc_compress that takes one of the rare routes on more than one block report MC_ERR_DEVICE while all its
 * kernels still end normally).  Applies to the calls issued afterwards.  Errors: MC_ERR_INVALID_ARG
 * (null, dense algorithm). */
int mc_set_barrier_spin_limit(mc_ctx *ctx, uint32_t polls);

/* Diagnostic for the sparsifiers (Top-k, DGC, Rand-k; Section 5.1 names their selection as the
 * costly step).  Synchronises the context's device and reports which route the exact
 * selection of the most recent mc_compress took:
 *   MC_SELECT_FAST    the threshold fell inside the histogram window kept from a margin below the
 *                     last threshold of this (group, worker) upward, in a bin of at most 4096 keys:
 *                     two short kernels after the streaming pass
 *   MC_SELECT_DENSE   as FAST, but more than 4096 keys share that bin (many equal values): the bin
 *                     is resolved as one more radix level
 *   MC_SELECT_ABOVE   the threshold rose above the window (also a context's first call of a
 *                     (group, worker)): three radix levels over the candidates
 *   MC_SELECT_REFILL  fewer than k elements passed the candidate filter: the group is
 *                     streamed a second time, every element a candidate
 * The last three run as one kernel with grid-wide barriers and cost several times the first
 * (measured on a 25.6 M element group: 60 / 160 / 180-260 / 410-450 us for the whole call).
 * The result of mc_compress is identical on all routes; only its cost differs.
 * Returns the route, or a negative mc_status (MC_ERR_INVALID_ARG for a dense algorithm). */
enum { MC_SELECT_ABOVE = 0, MC_SELECT_FAST = 1, MC_SELECT_REFILL = 2, MC_SELECT_DENSE = 3 };
int mc_last_select_route(mc_ctx *ctx);

/* Counts of mc_compress calls by the route their selection took (indexed by the MC_SELECT_ values) since
 * the context was created or the counts were last reset, for the sparsifiers without a sampled threshold;
 * and, of the most recent call, the number of keys that shared the threshold's window bin (the two-kernel
 * route lists them: at most 4096) and of elements that passed the candidate filter (modulo 2^32); and where the
 * candidate filter of that call's (group, worker) stands: the filter starts a margin below the last threshold,
 * 3/16 of an octave halved margin_halvings times (0..4: the library halves it while many more than k elements
 * pass, and starts over after a call whose threshold fell below the filter), at most margin_cap times for now
 * (4, less for a while after such a call).  -1 for both before the first call.
 * Synchronises the context's device.  Errors: MC_ERR_INVALID_ARG (null, dense algorithm). */
typedef struct {
    int64_t calls[4];
    int64_t last_bin_keys;
    int64_t last_candidates;
    int64_t margin_halvings;
    int64_t margin_cap;
} mc_select_counts;
int mc_select_stats(mc_ctx *ctx, mc_select_counts *out, int32_t reset);

/*
 * Per-kernel timing with HIP events recorded on the caller's stream around each
 * launch (off by default).  mc_profile_read synchronises the recorded events.
 *   mc_profile_select    bit i of the mask: time kernel slot i while enabled (default: all slots)
 *   mc_profile_kernels   number of kernel slots
 *   mc_profile_read      name (static string), launches and total milliseconds of slot `id`
 */
int mc_profile_enable(mc_ctx *ctx, int32_t on);
int mc_profile_select(mc_ctx *ctx, uint64_t kernel_mask);
int mc_profile_reset(mc_ctx *ctx);
int32_t mc_profile_kernels(void);
int mc_profile_read(mc_ctx *ctx, int32_t id, const char **name, int64_t *launches, double *total_ms);

const char *mc_strerror(int status);
const char *mc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MERGECOMP_H */
