/*
 * mc_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-threaded CPU statement of what MergeComp's per-group
 * compress / decompress-and-aggregate steps compute (Algorithm 1: delta = C(g),
 * g~ = aggregate(C^-1(Delta))), written to be checked against the paper by eye.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no source, header, table or helper with the HIP library.
 *
 * The paper names its compressors (Section 2.1, Table 1) but defines none of
 * them; each function below states the reading it follows.  All work on ONE
 * merged group: the flat fp32 vector obtained by concatenating the group's
 * tensors (Section 4.1: tensors of a group are merged and compressed in one
 * operation), so every scale, norm and top-k is per group.
 *
 * Arithmetic: fp32 element work is done in IEEE binary32 with one rounding per
 * operation (compile with -ffp-contract=off, no -ffast-math); reductions are
 * accumulated in fp64 in index order and rounded once.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors; top-k against a
 * library stable argsort and brute force; conservation payload + residual ==
 * gradient + old residual; exact-k; EF-Sign decode == scale*sign and the closed
 * form of the residual energy; unbiasedness of QSGD / TernGrad by averaging;
 * fp16 cast against a library cast; W=1 aggregate == decode; partition counts
 * against C(N-1, y-1) enumeration; the iteration-time model of the partition
 * search against closed forms (one group, free network, saturated network)
 * and a timeline worked by hand.  The four further schemes of Table 1: sign
 * planes against a library bit packer and scale invariance, the vote against a
 * library sign-of-sum, SigNUM with beta = 0 == SignSGD and the closed form of a
 * constant gradient, OneBit's two means against library means and the
 * least-squares property, Rand-k against a library stable argsort of the
 * pinned Philox draws, exact-k, value independence and uniformity.  Which
 * Philox counter and word every element of QSGD and TernGrad draws from
 * (worker, iteration, model-wide index: independent of the partition); the
 * directory that ends a sparse payload against a library searchsorted.  Parity of
 * absolute values with the paper is unpinned: the paper prints no compressor
 * input/output pair.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ALG_EFSIGN = 1, ALG_TOPK = 2, ALG_DGC = 3, ALG_QSGD = 4, ALG_TERNGRAD = 5, ALG_FP16 = 6,
       ALG_SIGNSGD = 7, ALG_SIGNUM = 8, ALG_ONEBIT = 9, ALG_RANDK = 10 };
enum { PART_EVEN_COUNT = 0, PART_EVEN_ELEMS = 1, PART_USER = 2 };

#define HDR_BYTES 128u   /* fields in the first 36 bytes, the rest zero: the body starts on a 128-byte line */
#define MAGIC 0x3150434Du /* "MCP1" */

typedef struct {
    int32_t algo;
    int32_t use_ef;        /* 1: p = g + e and e is updated; 0: p = g, state untouched */
    uint32_t ratio_ppm;    /* kept fraction of sparsifiers, parts per million */
    int32_t qsgd_bits;     /* code width incl. sign; levels s = 2^(bits-1) - 1 */
    float dgc_momentum;    /* m of DGC's momentum correction; beta of SigNUM */
    uint32_t sample_ppm;   /* DGC only: 0 = exact top-k; else the threshold is taken from a sample of this rate */
    uint64_t seed;         /* Philox key */
} orc_config;

/* ------------------------------------------------------------------------ */
/* Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter-based RNG.     */
/* ------------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod1;
        uint32_t n2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in [0,1) for one element.  Keying: key = seed; counter =
 * (J lo, J hi, worker, iter lo) with J = (model-global flat element index)/4,
 * output lane = index % 4.  The draw of an element therefore does not depend
 * on how the model is partitioned.  u = top 24 bits * 2^-24 (exact in fp32). */
float orc_uniform(uint64_t seed, uint32_t worker, uint64_t iter, uint64_t global_index)
{
    uint64_t J = global_index >> 2;
    uint32_t ctr[4] = { (uint32_t)J, (uint32_t)(J >> 32), worker, (uint32_t)iter };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    orc_philox4x32_10(ctr, key, r);
    return (float)(r[global_index & 3u] >> 8) * 5.9604644775390625e-8f; /* 2^-24 */
}

/* ------------------------------------------------------------------------ */
/* Partition (Section 4.3 notation: N tensors, y contiguous groups).          */
/* bounds[0]=0 < bounds[1] < ... < bounds[y]=N ; group j = [bounds[j],bounds[j+1]) */
/* ------------------------------------------------------------------------ */
int orc_partition(const int64_t *numel, int32_t N, int32_t y, int32_t policy,
                  const int32_t *user_bounds, int32_t *bounds)
{
    if (!numel || !bounds || N < 1 || y < 1) return -1;
    if (y > N) return -2;
    for (int t = 0; t < N; ++t) if (numel[t] < 0) return -1;
    if (policy == PART_EVEN_COUNT) {
        /* the paper's "naive" strategy (Section 5.2): even by tensor count */
        for (int j = 0; j <= y; ++j) bounds[j] = (int32_t)(((int64_t)j * N) / y);
    } else if (policy == PART_EVEN_ELEMS) {
        /* even by element count: boundary j is the smallest t whose prefix
         * reaches j/y of the model size D, then moved so no group is empty */
        int64_t D = 0;
        for (int t = 0; t < N; ++t) D += numel[t];
        bounds[0] = 0; bounds[y] = N;
        for (int j = 1; j < y; ++j) {
            int64_t prefix = 0; int t = 0;
            while (t < N && prefix * y < (int64_t)j * D) { prefix += numel[t]; ++t; }
            int lo = bounds[j - 1] + 1, hi = N - (y - j);
            if (t < lo) t = lo;
            if (t > hi) t = hi;
            bounds[j] = t;
        }
    } else if (policy == PART_USER) {
        if (!user_bounds) return -1;
        if (user_bounds[0] != 0 || user_bounds[y] != N) return -2;
        for (int j = 0; j < y; ++j) if (user_bounds[j + 1] <= user_bounds[j]) return -2;
        for (int j = 0; j <= y; ++j) bounds[j] = user_bounds[j];
    } else return -1;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Iteration time of a partition (Section 4.3): F(X_y) = A + sum h(x_i) +      */
/* sum g(x_i) - sum p(x_i) with linear h and g (Assumption 5).  The paper      */
/* gives no formula for the overlap p; it describes the schedule (wait-free    */
/* back-propagation, proof of Theorem 3), which is simulated here:             */
/*   - the GPU runs forward, then back-propagation tensor by tensor in list    */
/*     order (bwd[t] seconds each); when the last tensor of group i is done it  */
/*     compresses the group, h(x_i) = B_h + gamma_h x_i, then goes on;          */
/*   - the network sends group i for g(x_i) = B_g + gamma_g x_i seconds,        */
/*     starting when its compression is done and group i-1 has been sent.       */
/* F is the time at which the last group has been sent.                         */
/* ------------------------------------------------------------------------ */
typedef struct { double fwd, B_h, gamma_h, B_g, gamma_g; } orc_time_model;

int orc_partition_cost(const int64_t *numel, const double *bwd, int32_t N, const orc_time_model *m,
                       const int32_t *bounds, int32_t y, double *F)
{
    if (!numel || !bwd || !m || !bounds || !F || N < 1 || y < 1 || y > N) return -1;
    if (bounds[0] != 0 || bounds[y] != N) return -2;
    double gpu = m->fwd, net = 0.0;
    for (int i = 0; i < y; ++i) {
        if (bounds[i + 1] <= bounds[i]) return -2;
        int64_t x = 0;
        for (int t = bounds[i]; t < bounds[i + 1]; ++t) { gpu += bwd[t]; x += numel[t]; }
        gpu += m->B_h + m->gamma_h * (double)x;                  /* compress the group */
        double start = gpu > net ? gpu : net;                    /* the network may still be busy */
        net = start + (m->B_g + m->gamma_g * (double)x);
    }
    *F = net;
    return 0;
}

/* all partitions of N tensors into exactly y contiguous groups, the cheapest kept */
static void enumerate_partitions(const int64_t *numel, const double *bwd, int32_t N, const orc_time_model *m, int32_t y,
                                 int32_t *cur, int depth, double *bestF, int32_t *best)
{
    if (depth == y) {
        cur[y] = N;
        double F;
        if (orc_partition_cost(numel, bwd, N, m, cur, y, &F) == 0 && F < *bestF) {
            *bestF = F;
            memcpy(best, cur, (size_t)(y + 1) * sizeof(int32_t));
        }
        return;
    }
    /* boundary `depth` lies after boundary depth-1 and leaves a tensor for each later group */
    for (int32_t b = cur[depth - 1] + 1; b <= N - (y - depth); ++b) {
        cur[depth] = b;
        enumerate_partitions(numel, bwd, N, m, y, cur, depth + 1, bestF, best);
    }
}

/* F_min(y) and one partition that attains it, by trying all C(N-1, y-1) (Lemma 1) */
int orc_partition_best(const int64_t *numel, const double *bwd, int32_t N, const orc_time_model *m, int32_t y,
                       int32_t *bounds, double *F)
{
    if (y < 1 || y > N || N > 24) return -2;
    int32_t cur[26];
    double bestF = INFINITY;
    cur[0] = 0;
    enumerate_partitions(numel, bwd, N, m, y, cur, 1, &bestF, bounds);
    *F = bestF;
    return 0;
}

/* The heuristic of Algorithm 2: grow y from 2; stop at y-1 as soon as the best y groups are slower
 * than the best y-1, stop at y as soon as the gain drops below alpha * F_min(y-1), else end at Y. */
int orc_partition_search(const int64_t *numel, const double *bwd, int32_t N, const orc_time_model *m, int32_t Y,
                         double alpha, int32_t *bounds, int32_t *y_out, double *F_out)
{
    if (Y < 1 || N > 24) return -2;
    if (Y > N) Y = N;
    int32_t prev[26], now[26];
    double Fprev, Fnow;
    orc_partition_best(numel, bwd, N, m, 1, prev, &Fprev);
    int32_t ybest = 1;
    for (int32_t y = 2; y <= Y; ++y) {
        orc_partition_best(numel, bwd, N, m, y, now, &Fnow);
        if (Fprev < Fnow) break;                                   /* more groups made it worse: keep y-1 */
        int stop = Fprev - Fnow < alpha * Fprev;                   /* marginal benefit too small: keep y, stop */
        memcpy(prev, now, (size_t)(y + 1) * sizeof(int32_t));
        Fprev = Fnow; ybest = y;
        if (stop) break;
    }
    memcpy(bounds, prev, (size_t)(ybest + 1) * sizeof(int32_t));
    *y_out = ybest; *F_out = Fprev;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* sizes                                                                      */
/* ------------------------------------------------------------------------ */
/* kept count of a sparsifier: k = max(1, floor(n*ppm/1e6)), capped at n */
int64_t orc_topk_count(int64_t n, uint32_t ppm)
{
    if (n <= 0) return 0;
    int64_t k = (int64_t)(((__int128)n * ppm) / 1000000);
    if (k < 1) k = 1;
    if (k > n) k = n;
    return k;
}

/* entries a sparse payload has room for: k, or twice k (at most n) when DGC estimates its threshold
 * from a sample and the number of kept entries varies from call to call */
int64_t orc_sparse_capacity(const orc_config *c, int64_t n)
{
    int64_t k = orc_topk_count(n, c->ratio_ppm);
    if (c->algo == ALG_DGC && c->sample_ppm) { k *= 2; if (k > n) k = n; }
    return k;
}

/* A sparse payload ends with a directory of its ascending index list: entry t counts the kept entries whose
 * index lies below t * DIR_SPAN, for t = 0 .. ceil(n / DIR_SPAN) (so the first is 0 and the last the number of
 * kept entries; an empty group has no directory).  It adds nothing to what the payload says; a receiver that sums
 * many such lists span by span finds each list's share of a span without searching.  (Wire layout, which the paper
 * leaves open.) */
#define DIR_SPAN 4096
int64_t orc_dir_spans(int64_t n) { return (n + DIR_SPAN - 1) / DIR_SPAN; }
static void put_directory(uint8_t *payload, int64_t n, int64_t cap, const uint32_t *idx, int64_t kept)
{
    if (n <= 0) return;
    uint32_t *dir = (uint32_t *)(payload + HDR_BYTES + 8 * cap);
    int64_t j = 0;
    for (int64_t t = 0; t <= orc_dir_spans(n); ++t) {
        while (j < kept && (int64_t)idx[j] < t * DIR_SPAN) ++j;
        dir[t] = (uint32_t)j;
    }
}

static int64_t words32(int64_t n) { return (n + 31) / 32; }
static int64_t pad4(int64_t b) { return (b + 3) / 4 * 4; }

int64_t orc_payload_bytes(const orc_config *c, int64_t n)
{
    switch (c->algo) {
    case ALG_EFSIGN:
    case ALG_SIGNSGD:
    case ALG_SIGNUM:
    case ALG_ONEBIT:   return HDR_BYTES + 4 * words32(n);
    case ALG_TERNGRAD: return HDR_BYTES + 8 * words32(n);
    case ALG_QSGD:     return HDR_BYTES + pad4(n);
    case ALG_FP16:     return HDR_BYTES + pad4(2 * n);
    case ALG_TOPK:
    case ALG_DGC:
    case ALG_RANDK:    return HDR_BYTES + 8 * orc_sparse_capacity(c, n) + (n > 0 ? 4 * (orc_dir_spans(n) + 1) : 0);
    }
    return -1;
}

/* floats of per-group memory: residual e (DGC: v then u; SigNUM: the momentum; SignSGD: none) */
int64_t orc_state_floats(const orc_config *c, int64_t n)
{
    if (c->algo == ALG_SIGNSGD) return 0;
    return c->algo == ALG_DGC ? 2 * n : n;
}

static void put_header(uint8_t *payload, int32_t algo, int64_t n, int64_t k, float scale, uint32_t levels)
{
    uint32_t magic = MAGIC, a = (uint32_t)algo;
    uint64_t nn = (uint64_t)n, kk = (uint64_t)k;
    memset(payload, 0, HDR_BYTES);
    memcpy(payload + 0, &magic, 4);
    memcpy(payload + 4, &a, 4);
    memcpy(payload + 8, &nn, 8);
    memcpy(payload + 16, &kk, 8);
    memcpy(payload + 24, &scale, 4);
    memcpy(payload + 28, &levels, 4);
}

/* ------------------------------------------------------------------------ */
/* binary32 -> binary16, round to nearest even; overflow -> inf; subnormals    */
/* kept; NaN stays NaN (quiet).  Written out on the bit patterns.             */
/* ------------------------------------------------------------------------ */
static uint16_t f32_to_f16_rne(float x)
{
    uint32_t b; memcpy(&b, &x, 4);
    uint16_t sign = (uint16_t)((b >> 16) & 0x8000u);
    uint32_t expo = (b >> 23) & 0xFFu;
    uint32_t man = b & 0x7FFFFFu;
    if (expo == 0xFFu) return (uint16_t)(sign | 0x7C00u | (man ? 0x200u | (man >> 13) : 0u));
    int32_t e = (int32_t)expo - 127 + 15;            /* biased half exponent */
    if (e >= 31) return (uint16_t)(sign | 0x7C00u);  /* too large: inf */
    uint32_t sig, shift;
    if (e >= 1) { sig = man; shift = 13; }           /* normal half */
    else {
        if (e < -10) return sign;                    /* below half of the smallest subnormal */
        sig = man | 0x800000u;                       /* make the hidden bit explicit */
        shift = (uint32_t)(14 - e);                  /* 14..24 */
        e = 0;
    }
    uint32_t kept = sig >> shift;
    uint32_t rest = sig & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    uint32_t h = ((uint32_t)e << 10) + kept;         /* a carry out of the mantissa bumps the exponent */
    if (rest > half || (rest == half && (kept & 1u))) h += 1u;
    return (uint16_t)(sign | h);
}

static float f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t expo = (h >> 10) & 0x1Fu, man = h & 0x3FFu, b;
    if (expo == 0x1Fu) b = sign | 0x7F800000u | (man << 13);
    else if (expo) b = sign | ((expo - 15 + 127) << 23) | (man << 13);
    else if (!man) b = sign;
    else { /* subnormal half: value = man * 2^-24 */
        float v = (float)man * 5.9604644775390625e-8f;
        memcpy(&b, &v, 4); b |= sign;
    }
    float f; memcpy(&f, &b, 4); return f;
}

void orc_f32_to_f16(const float *x, uint16_t *h, int64_t n) { for (int64_t i = 0; i < n; ++i) h[i] = f32_to_f16_rne(x[i]); }
void orc_f16_to_f32(const uint16_t *h, float *x, int64_t n) { for (int64_t i = 0; i < n; ++i) x[i] = f16_to_f32(h[i]); }

/* ------------------------------------------------------------------------ */
/* exact top-k of |p| with "lower index wins" on ties                         */
/* ------------------------------------------------------------------------ */
typedef struct { uint32_t key; uint32_t idx; } keyidx;

static int cmp_key_desc_idx_asc(const void *a, const void *b)
{
    const keyidx *x = (const keyidx *)a, *y = (const keyidx *)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1;
    if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
    return 0;
}

/* The 31-bit selection key of Rand-k: the element's Philox word (same counter layout as
 * orc_uniform) without its lowest bit.  Taking the k largest keys picks k distinct
 * positions uniformly at random, whatever the values are. */
uint32_t orc_randk_key(uint64_t seed, uint32_t worker, uint64_t iter, uint64_t global_index)
{
    uint64_t J = global_index >> 2;
    uint32_t ctr[4] = { (uint32_t)J, (uint32_t)(J >> 32), worker, (uint32_t)iter };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t r[4];
    orc_philox4x32_10(ctr, key, r);
    return r[global_index & 3u] >> 1;
}

/* selected[i] = 1 for the k elements that come first when all elements are
 * ordered by (key descending, index ascending).  Top-k / DGC: key = |p| compared on
 * the bit pattern with the sign cleared, which orders finite fp32 magnitudes
 * (rk = NULL).  Rand-k: key = rk[i]. */
static int select_topk(const float *p, const uint32_t *rk, int64_t n, int64_t k, uint8_t *selected)
{
    keyidx *a = (keyidx *)malloc((size_t)(n > 0 ? n : 1) * sizeof(keyidx));
    if (!a) return -3;
    for (int64_t i = 0; i < n; ++i) {
        uint32_t b; memcpy(&b, &p[i], 4);
        a[i].key = rk ? rk[i] : (b & 0x7FFFFFFFu); a[i].idx = (uint32_t)i;
    }
    qsort(a, (size_t)n, sizeof(keyidx), cmp_key_desc_idx_asc);
    memset(selected, 0, (size_t)n);
    for (int64_t j = 0; j < k; ++j) selected[a[j].idx] = 1;
    free(a);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* compress one group                                                         */
/*   g[n]        gradient of the group (flat)                                 */
/*   state       error-feedback memory: e[n]  (DGC: v[n] then u[n])           */
/*   payload     out, orc_payload_bytes() bytes                               */
/*   group_off   model-global flat index of the group's element 0 (RNG only)   */
/*   scale_in    NULL, or the group scalar(s) to encode with instead of the    */
/*               ones computed here (EF-Sign scale, QSGD norm, TernGrad max;   */
/*               OneBit: two floats, the means); used by parity tests once the */
/*               scalars themselves have been checked                          */
/*   scale_out   NULL, or receives the scalar(s) computed here (OneBit: two)   */
/* ------------------------------------------------------------------------ */
int orc_compress(const orc_config *c, int64_t n, uint64_t group_off, uint32_t worker, uint64_t iter,
                 const float *g, float *state, uint8_t *payload, const float *scale_in, float *scale_out)
{
    if (!c || !payload || n < 0 || (n > 0 && !g)) return -1;
    if (n >= ((int64_t)1 << 32)) return -2;
    if (c->algo == ALG_SIGNSGD && c->use_ef) return -1;             /* plain signs: nothing is remembered */
    if ((c->algo == ALG_SIGNUM || c->algo == ALG_RANDK) && !c->use_ef) return -1;   /* these always carry state */
    const int ef = c->use_ef != 0;
    if (ef && n > 0 && !state) return -1;
    memset(payload, 0, (size_t)orc_payload_bytes(c, n));
    if (scale_out) *scale_out = 0.0f;

    /* DGC has its own accumulate step; everything else: p = g (+ e) */
    float *p = (float *)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
    if (!p) return -3;
    if (c->algo == ALG_DGC) {
        /* momentum correction: u = m*u + g ; v = v + u ; the vector compressed is v */
        if (!ef) { free(p); return -1; }
        float *v = state, *u = state + n;
        for (int64_t i = 0; i < n; ++i) {
            float mu = c->dgc_momentum * u[i];
            u[i] = mu + g[i];
            v[i] = v[i] + u[i];
            p[i] = v[i];
        }
    } else if (c->algo == ALG_SIGNUM) {
        /* the vector whose signs are sent is the momentum m = beta*m + (1 - beta)*g */
        const float beta = c->dgc_momentum, omb = 1.0f - beta;
        for (int64_t i = 0; i < n; ++i) {
            float bm = beta * state[i], og = omb * g[i];
            state[i] = bm + og;
            p[i] = state[i];
        }
    } else {
        for (int64_t i = 0; i < n; ++i) p[i] = ef ? g[i] + state[i] : g[i];
    }

    int rc = 0;
    switch (c->algo) {
    case ALG_EFSIGN: {
        /* delta = (||p||_1 / n) * sign(p), sign(0) = +1 ; e = p - delta */
        double S = 0.0;
        for (int64_t i = 0; i < n; ++i) S += fabs((double)p[i]);
        float scale = n > 0 ? (float)(S / (double)n) : 0.0f;
        if (scale_out) *scale_out = scale;
        if (scale_in) scale = *scale_in;
        put_header(payload, c->algo, n, 0, scale, 0);
        uint32_t *w = (uint32_t *)(payload + HDR_BYTES);
        for (int64_t i = 0; i < n; ++i) {
            int bit = p[i] >= 0.0f;
            if (bit) w[i / 32] |= 1u << (i % 32);
            float d = bit ? scale : -scale;
            if (ef) state[i] = p[i] - d;
        }
        break;
    }
    case ALG_SIGNSGD:
    case ALG_SIGNUM: {
        /* delta = sign(p), sign(0) = +1: one bit per element, decoded as +-1; no residual
         * (SignSGD: p = g; SigNUM: p = momentum, updated above) */
        put_header(payload, c->algo, n, 0, 1.0f, 0);
        uint32_t *w = (uint32_t *)(payload + HDR_BYTES);
        for (int64_t i = 0; i < n; ++i) if (p[i] >= 0.0f) w[i / 32] |= 1u << (i % 32);
        break;
    }
    case ALG_ONEBIT: {
        /* one bit per element, reconstructed as the mean of its class: mu+ over the
         * elements with p >= 0, mu- over those with p < 0 ; e = p - delta */
        double Sp = 0.0, Sn = 0.0; int64_t np = 0;
        for (int64_t i = 0; i < n; ++i) { if (p[i] >= 0.0f) { Sp += (double)p[i]; ++np; } else Sn += (double)p[i]; }
        float mu[2];
        mu[0] = np > 0 ? (float)(Sp / (double)np) : 0.0f;
        mu[1] = n - np > 0 ? (float)(Sn / (double)(n - np)) : 0.0f;
        if (scale_out) { scale_out[0] = mu[0]; scale_out[1] = mu[1]; }
        if (scale_in) { mu[0] = scale_in[0]; mu[1] = scale_in[1]; }
        put_header(payload, c->algo, n, 0, mu[0], 0);
        memcpy(payload + 32, &mu[1], 4);                 /* second scalar right after the common fields */
        uint32_t *w = (uint32_t *)(payload + HDR_BYTES);
        for (int64_t i = 0; i < n; ++i) {
            int bit = p[i] >= 0.0f;
            if (bit) w[i / 32] |= 1u << (i % 32);
            float d = bit ? mu[0] : mu[1];
            if (ef) state[i] = p[i] - d;
        }
        break;
    }
    case ALG_TOPK:
    case ALG_DGC:
    case ALG_RANDK: {
        if (c->algo == ALG_DGC && c->sample_ppm) {
            /* DGC's cheaper selection: instead of the exact top-k of all n values, take the threshold
             * that keeps the given ratio of a SAMPLE and send everything that reaches it.
             *   sample      every stride-th element, stride = floor(1e6 / sample_ppm), starting at a
             *               Philox-drawn offset (the word of the group's first element, see orc_uniform)
             *   threshold   the ks-th largest key of the sample, ks = max(1, floor(m ratio)), m = sample size
             *   kept        keys above the threshold, then keys equal to it, each in index order, until the
             *               payload's capacity cap = min(n, 2k) is reached; the header's k is the count kept and
             *               its levels field names the capacity (the values start after cap indices)
             * unused payload entries stay zero; kept entries leave both accumulators. */
            const int64_t cap = orc_sparse_capacity(c, n);
            uint32_t stride = 1000000u / c->sample_ppm; if (stride < 1) stride = 1;
            uint64_t J = group_off >> 2;
            uint32_t ctr[4] = { (uint32_t)J, (uint32_t)(J >> 32), worker, (uint32_t)iter };
            uint32_t key2[2] = { (uint32_t)c->seed, (uint32_t)(c->seed >> 32) }, r[4];
            orc_philox4x32_10(ctr, key2, r);
            const uint32_t first = r[group_off & 3u] % stride;
            int64_t m = 0;
            for (int64_t i = first; i < n; i += stride) ++m;
            uint32_t thr = 0;                                   /* empty sample: everything reaches the threshold */
            if (m > 0) {
                keyidx *smp = (keyidx *)malloc((size_t)m * sizeof(keyidx));
                if (!smp) { rc = -3; break; }
                int64_t j = 0;
                for (int64_t i = first; i < n; i += stride, ++j) {
                    uint32_t bb; memcpy(&bb, &p[i], 4);
                    smp[j].key = bb & 0x7FFFFFFFu; smp[j].idx = (uint32_t)i;
                }
                qsort(smp, (size_t)m, sizeof(keyidx), cmp_key_desc_idx_asc);
                int64_t ks = (int64_t)(((__int128)m * c->ratio_ppm) / 1000000);
                if (ks < 1) ks = 1;
                thr = smp[ks - 1].key;
                free(smp);
            }
            uint32_t *idx = (uint32_t *)(payload + HDR_BYTES);
            float *val = (float *)(payload + HDR_BYTES + 4 * cap);
            uint8_t *sel = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
            if (!sel) { rc = -3; break; }
            int64_t kept = 0;
            for (int pass = 0; pass < 2; ++pass)                /* above the threshold first, then equal to it */
                for (int64_t i = 0; i < n && kept < cap; ++i) {
                    uint32_t bb; memcpy(&bb, &p[i], 4); bb &= 0x7FFFFFFFu;
                    if (pass == 0 ? bb > thr : bb == thr) { sel[i] = 1; ++kept; }
                }
            put_header(payload, c->algo, n, kept, 0.0f, (uint32_t)cap);   /* the capacity travels in the header */
            int64_t j = 0;
            float *v = state, *u = state + n;
            for (int64_t i = 0; i < n; ++i)
                if (sel[i]) { idx[j] = (uint32_t)i; val[j] = p[i]; ++j; v[i] = 0.0f; u[i] = 0.0f; }
            put_directory(payload, n, cap, idx, kept);
            free(sel);
            break;
        }
        int64_t k = orc_topk_count(n, c->ratio_ppm);
        uint8_t *sel = (uint8_t *)malloc((size_t)(n > 0 ? n : 1));
        if (!sel) { rc = -3; break; }
        uint32_t *rk = NULL;
        if (c->algo == ALG_RANDK) {
            /* k positions chosen uniformly at random (independent of the values): the k largest Philox keys */
            rk = (uint32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(uint32_t));
            if (!rk) { free(sel); rc = -3; break; }
            for (int64_t i = 0; i < n; ++i) rk[i] = orc_randk_key(c->seed, worker, iter, group_off + (uint64_t)i);
        }
        rc = select_topk(p, rk, n, k, sel);
        free(rk);
        if (rc) { free(sel); break; }
        put_header(payload, c->algo, n, k, 0.0f, 0);
        uint32_t *idx = (uint32_t *)(payload + HDR_BYTES);
        float *val = (float *)(payload + HDR_BYTES + 4 * k);
        int64_t j = 0;
        for (int64_t i = 0; i < n; ++i) {           /* ascending index order */
            if (sel[i]) { idx[j] = (uint32_t)i; val[j] = p[i]; ++j; }
        }
        put_directory(payload, n, k, idx, k);
        if (c->algo == ALG_DGC) {
            /* selected entries leave both accumulators (momentum factor masking) */
            float *v = state, *u = state + n;
            for (int64_t i = 0; i < n; ++i) if (sel[i]) { v[i] = 0.0f; u[i] = 0.0f; }
        } else if (ef) {
            for (int64_t i = 0; i < n; ++i) state[i] = sel[i] ? 0.0f : p[i];
        }
        free(sel);
        break;
    }
    case ALG_QSGD: {
        /* delta_i = ||p||_2 * sgn(p_i) * xi_i / s, xi_i = floor(a_i) + [u_i < frac(a_i)],
         * a_i = |p_i| * s / ||p||_2 : stochastic rounding to one of s+1 levels */
        if (c->qsgd_bits < 2 || c->qsgd_bits > 8) { rc = -1; break; }
        const int s = (1 << (c->qsgd_bits - 1)) - 1;
        double S = 0.0;
        for (int64_t i = 0; i < n; ++i) S += (double)p[i] * (double)p[i];
        float norm = (float)sqrt(S);
        if (scale_out) *scale_out = norm;
        if (scale_in) norm = *scale_in;
        put_header(payload, c->algo, n, 0, norm, (uint32_t)s);
        int8_t *code = (int8_t *)(payload + HDR_BYTES);
        const float sf = (float)s;
        const float r = norm > 0.0f ? sf / norm : 0.0f;     /* one fp32 divide per group */
        const float q = norm / sf;                          /* decode step */
        for (int64_t i = 0; i < n; ++i) {
            int xi = 0;
            if (norm > 0.0f) {
                float a = fabsf(p[i]) * r;
                if (a < sf) {
                    float l = floorf(a);
                    float f = a - l;
                    float u = orc_uniform(c->seed, worker, iter, group_off + (uint64_t)i);
                    xi = (int)l + (u < f ? 1 : 0);
                    if (xi > s) xi = s;
                } else xi = s;
            }
            int cd = p[i] < 0.0f ? -xi : xi;
            code[i] = (int8_t)cd;
            float d = (float)cd * q;
            if (ef) state[i] = p[i] - d;
        }
        break;
    }
    case ALG_TERNGRAD: {
        /* delta_i = smax * sgn(p_i) * b_i, b_i ~ Bernoulli(|p_i| / smax), smax = max|p|;
         * the Bernoulli draw is taken division-free as [u_i * smax < |p_i|] */
        float smax = 0.0f;
        for (int64_t i = 0; i < n; ++i) { float a = fabsf(p[i]); if (a > smax) smax = a; }
        if (scale_out) *scale_out = smax;
        if (scale_in) smax = *scale_in;
        put_header(payload, c->algo, n, 0, smax, 0);
        uint32_t *nzp = (uint32_t *)(payload + HDR_BYTES);
        uint32_t *ngp = nzp + words32(n);
        for (int64_t i = 0; i < n; ++i) {
            float u = orc_uniform(c->seed, worker, iter, group_off + (uint64_t)i);
            int nz = (u * smax) < fabsf(p[i]);
            int neg = nz && p[i] < 0.0f;
            if (nz) nzp[i / 32] |= 1u << (i % 32);
            if (neg) ngp[i / 32] |= 1u << (i % 32);
            float d = nz ? (neg ? -smax : smax) : 0.0f;
            if (ef) state[i] = p[i] - d;
        }
        break;
    }
    case ALG_FP16: {
        put_header(payload, c->algo, n, 0, 0.0f, 0);
        uint16_t *h = (uint16_t *)(payload + HDR_BYTES);
        for (int64_t i = 0; i < n; ++i) {
            h[i] = f32_to_f16_rne(p[i]);
            float d = f16_to_f32(h[i]);
            if (ef) state[i] = p[i] - d;
        }
        break;
    }
    default: rc = -1;
    }
    free(p);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* decode one payload into a dense vector d[n] (what C^-1 reconstructs)        */
/* ------------------------------------------------------------------------ */
int orc_decode(const uint8_t *payload, int64_t n, float *d)
{
    uint32_t magic, algo, levels; uint64_t pn, k; float scale;
    memcpy(&magic, payload, 4); memcpy(&algo, payload + 4, 4); memcpy(&pn, payload + 8, 8);
    memcpy(&k, payload + 16, 8); memcpy(&scale, payload + 24, 4); memcpy(&levels, payload + 28, 4);
    if (magic != MAGIC || (int64_t)pn != n) return -5;
    const uint8_t *body = payload + HDR_BYTES;
    switch (algo) {
    case ALG_EFSIGN: {
        const uint32_t *w = (const uint32_t *)body;
        for (int64_t i = 0; i < n; ++i) d[i] = ((w[i / 32] >> (i % 32)) & 1u) ? scale : -scale;
        break;
    }
    case ALG_SIGNSGD:
    case ALG_SIGNUM: {
        const uint32_t *w = (const uint32_t *)body;
        for (int64_t i = 0; i < n; ++i) d[i] = ((w[i / 32] >> (i % 32)) & 1u) ? 1.0f : -1.0f;
        break;
    }
    case ALG_ONEBIT: {
        float lo; memcpy(&lo, payload + 32, 4);
        const uint32_t *w = (const uint32_t *)body;
        for (int64_t i = 0; i < n; ++i) d[i] = ((w[i / 32] >> (i % 32)) & 1u) ? scale : lo;
        break;
    }
    case ALG_TOPK:
    case ALG_DGC:
    case ALG_RANDK: {
        const uint32_t *idx = (const uint32_t *)body;
        /* values follow the index array, whose length is k, or the capacity named in the header (sampled DGC) */
        const float *val = (const float *)(body + 4 * (levels ? (uint64_t)levels : k));
        for (int64_t i = 0; i < n; ++i) d[i] = 0.0f;
        for (uint64_t j = 0; j < k; ++j) { if (idx[j] >= (uint64_t)n) return -5; d[idx[j]] = val[j]; }
        break;
    }
    case ALG_QSGD: {
        const int8_t *code = (const int8_t *)body;
        const float q = scale / (float)levels;
        for (int64_t i = 0; i < n; ++i) d[i] = (float)code[i] * q;
        break;
    }
    case ALG_TERNGRAD: {
        const uint32_t *nzp = (const uint32_t *)body, *ngp = nzp + words32(n);
        for (int64_t i = 0; i < n; ++i) {
            int nz = (nzp[i / 32] >> (i % 32)) & 1u, neg = (ngp[i / 32] >> (i % 32)) & 1u;
            d[i] = nz ? (neg ? -scale : scale) : 0.0f;
        }
        break;
    }
    case ALG_FP16: {
        const uint16_t *h = (const uint16_t *)body;
        for (int64_t i = 0; i < n; ++i) d[i] = f16_to_f32(h[i]);
        break;
    }
    default: return -5;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* aggregate: out = alpha * (((0 + d_0) + d_1) + ... + d_{W-1}), fp32, workers */
/* in ascending order (Algorithm 1: g~ = aggregate(C^-1(Delta))).              */
/* SignSGD / SigNUM aggregate by majority vote: the sum of the +-1 becomes its */
/* sign (-1, 0 on a tie, +1) before alpha is applied.                          */
/* ------------------------------------------------------------------------ */
int orc_decompress_sum(int64_t n, const uint8_t *const *payloads, int32_t W, float alpha, float *out)
{
    if (n < 0 || W < 1 || !payloads || (n > 0 && !out)) return -1;
    float *d = (float *)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
    if (!d) return -3;
    for (int64_t i = 0; i < n; ++i) out[i] = 0.0f;
    for (int w = 0; w < W; ++w) {
        int rc = orc_decode(payloads[w], n, d);
        if (rc) { free(d); return rc; }
        for (int64_t i = 0; i < n; ++i) out[i] = out[i] + d[i];
    }
    uint32_t algo; memcpy(&algo, payloads[0] + 4, 4);
    if (algo == ALG_SIGNSGD || algo == ALG_SIGNUM)
        for (int64_t i = 0; i < n; ++i) out[i] = out[i] > 0.0f ? 1.0f : (out[i] < 0.0f ? -1.0f : 0.0f);
    for (int64_t i = 0; i < n; ++i) out[i] = alpha * out[i];
    free(d);
    return 0;
}
