/*
 * Pipe-SGD aggregation + update: CPU ORACLE.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, scalar, obviously-correct
 * statement of what the hot path computes. Only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg may use it. The product (the HIP
 * library) shares no code with it and never calls it.
 *
 * What it follows (arXiv 1811.03619):
 *   - Sec. 3.1, Ring-AllReduce paragraph + Fig. 2(c): every worker transmits
 *     one block of the gradient to its ring neighbour and sum-reduces the
 *     block it receives (p-1 rounds of transmitting and reducing), until each block
 *     is fully reduced on a different worker; the reduced blocks then travel
 *     round the ring to the other workers (p-1 more rounds).  Cost terms of
 *     Eq. 5: 2(p-1) rounds, 2((p-1)/p)n bytes sent, ((p-1)/p)n bytes reduced.
 *   - Sec. 3.2: truncation (drop low mantissa bits, 16 bits kept) and scalar
 *     quantization (8-bit integers, range set by the largest magnitude);
 *     (decompress, sum, compress) at every transmit-and-reduce round.
 *   - Algorithm 1, compute thread lines 4-5: decompress the aggregated
 *     gradient of iteration t-K, then w[t] = w[t-1] - gamma * g_sum[t-K].
 *
 * Readings taken where the paper is silent:
 *   ring direction r -> r+1; block c starts its sum on worker c; the local
 *   operand of every sum is the worker's full-precision fp32 block; the
 *   send-back rounds forward the compressed block verbatim; truncation keeps
 *   the top 16 bits (toward zero); quantization blocks are 4096 consecutive
 *   elements, scale = max|x|, inv = 127/scale (saturated at FLT_MAX),
 *   q = rint(x*inv) clamped to [-127,127] (ties to even), dequantised value
 *   = q * (scale/127); momentum form v = m*v + g, w = w - lr*v with single
 *   rounding per fused multiply-add.
 *
 * Arithmetic is IEEE-754 binary32 throughout (the precision the workload
 * fixes); build with -ffp-contract=off and without fast-math so that every
 * operation written below is exactly one rounding.
 *
 * Two more schedules with the same result definition follow the ring
 * section: the one-exchange "direct" AllReduce and recursive halving and
 * doubling.
 *
 * Pinned by tests/test_oracle_*.py (closed forms, invariants, exhaustive
 * codec sweeps, hand-worked tiny cases; tests/test_oracle_mutants.py checks
 * that planted mistakes trip them).  Parity unpinned: nothing exported
 * here lacks a pin; the *choices* listed above are readings, not facts of the
 * paper.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_NONE = 0, ORC_TRUNC16 = 1, ORC_QUANT8 = 2 };
#define ORC_QBLOCK 4096u

/* ---------------------------------------------------------------- sizes -- */

/* Block ("chunk") length used to split an n-element vector over p workers:
 * ceil(n/p) rounded up to a whole number of quantization blocks, so that no
 * quantization block straddles two ring blocks.  (Sec. 3.1 gives every worker
 * one block of the gradient vector; n/p in Eq. 5.) */
size_t orc_chunk_elems(size_t n, int p)
{
    size_t per = (n + (size_t)p - 1) / (size_t)p;
    return (per + ORC_QBLOCK - 1) / ORC_QBLOCK * ORC_QBLOCK;
}

static size_t chunk_lo(size_t n, size_t ce, int c)
{
    size_t lo = (size_t)c * ce;
    return lo < n ? lo : n;
}
static size_t chunk_hi(size_t n, size_t ce, int c)
{
    size_t hi = ((size_t)c + 1) * ce;
    return hi < n ? hi : n;
}

size_t orc_payload_bytes(int mode, size_t n)
{
    switch (mode) {
    case ORC_NONE:    return 4 * n;
    case ORC_TRUNC16: return 2 * n;
    case ORC_QUANT8:  return n;
    }
    return 0;
}
size_t orc_num_scales(int mode, size_t n)
{
    return mode == ORC_QUANT8 ? (n + ORC_QBLOCK - 1) / ORC_QBLOCK : 0;
}

/* --------------------------------------------------------------- codecs -- */

static uint32_t f2u(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
static float    u2f(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }

/* Truncation (Sec. 3.2): keep sign, exponent and the 7 leading mantissa
 * bits; the 16 trailing mantissa bits are dropped. */
static uint16_t trunc16_c(float x) { return (uint16_t)(f2u(x) >> 16); }
static float    trunc16_d(uint16_t h) { return u2f((uint32_t)h << 16); }

/* Scalar quantization (Sec. 3.2) of one block of up to 4096 values. */
static float quant8_block_c(const float *x, size_t len, int8_t *q)
{
    float scale = 0.0f;
    for (size_t i = 0; i < len; ++i) {
        float a = fabsf(x[i]);
        if (a > scale) scale = a;
    }
    if (scale == 0.0f) {
        for (size_t i = 0; i < len; ++i) q[i] = 0;
        return 0.0f;
    }
    float inv = 127.0f / scale;
    if (inv > FLT_MAX) inv = FLT_MAX;
    for (size_t i = 0; i < len; ++i) {
        float t = x[i] * inv;
        float r = rintf(t);            /* default rounding mode: ties to even */
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        q[i] = (int8_t)r;
    }
    return scale;
}
static void quant8_block_d(const int8_t *q, float scale, size_t len, float *x)
{
    float step = scale / 127.0f;
    for (size_t i = 0; i < len; ++i) x[i] = (float)q[i] * step;
}

void orc_compress(int mode, const float *x, size_t n, void *payload, float *scales)
{
    if (mode == ORC_NONE) {
        float *o = (float *)payload;
        for (size_t i = 0; i < n; ++i) o[i] = x[i];
    } else if (mode == ORC_TRUNC16) {
        uint16_t *o = (uint16_t *)payload;
        for (size_t i = 0; i < n; ++i) o[i] = trunc16_c(x[i]);
    } else {
        int8_t *o = (int8_t *)payload;
        for (size_t b = 0, i = 0; i < n; ++b, i += ORC_QBLOCK) {
            size_t len = n - i < ORC_QBLOCK ? n - i : ORC_QBLOCK;
            scales[b] = quant8_block_c(x + i, len, o + i);
        }
    }
}

void orc_decompress(int mode, const void *payload, const float *scales, size_t n, float *x)
{
    if (mode == ORC_NONE) {
        const float *in = (const float *)payload;
        for (size_t i = 0; i < n; ++i) x[i] = in[i];
    } else if (mode == ORC_TRUNC16) {
        const uint16_t *in = (const uint16_t *)payload;
        for (size_t i = 0; i < n; ++i) x[i] = trunc16_d(in[i]);
    } else {
        const int8_t *in = (const int8_t *)payload;
        for (size_t b = 0, i = 0; i < n; ++b, i += ORC_QBLOCK) {
            size_t len = n - i < ORC_QBLOCK ? n - i : ORC_QBLOCK;
            quant8_block_d(in + i, scales[b], len, x + i);
        }
    }
}

/* ------------------------------------------------------- ring simulator -- */

/* One message on the wire: a compressed block. */
typedef struct {
    int    chunk;          /* which block of the vector it carries */
    size_t len;            /* elements */
    void  *payload;        /* orc_payload_bytes(mode, len) */
    float *scales;         /* orc_num_scales(mode, len) */
} orc_msg;

typedef struct {
    int     mode, p;
    size_t  n, ce;
    float **work;          /* p working vectors: start as the local gradients;
                              a block is overwritten by the partial sum when
                              the worker reduces into it */
    orc_msg *wire;         /* p in-flight messages, wire[r] = sent by worker r */
    void  **res_payload;   /* p result slots: the aggregated gradient in
                              compressed format (Alg. 1, g^c_sum) */
    float **res_scales;
    /* bookkeeping for the Eq. 5 coefficients */
    int      rounds;
    uint64_t *elems_sent, *elems_reduced, *bytes_sent;
    float   *tmp;          /* one decompressed block */
} orc_ring;

static int modp(int a, int p) { int m = a % p; return m < 0 ? m + p : m; }

orc_ring *orc_ring_new(int mode, int p, size_t n, const float *const *g_local)
{
    orc_ring *R = (orc_ring *)calloc(1, sizeof *R);
    R->mode = mode; R->p = p; R->n = n; R->ce = orc_chunk_elems(n, p);
    R->work = (float **)calloc((size_t)p, sizeof(float *));
    R->wire = (orc_msg *)calloc((size_t)p, sizeof(orc_msg));
    R->res_payload = (void **)calloc((size_t)p, sizeof(void *));
    R->res_scales = (float **)calloc((size_t)p, sizeof(float *));
    R->elems_sent = (uint64_t *)calloc((size_t)p, 8);
    R->elems_reduced = (uint64_t *)calloc((size_t)p, 8);
    R->bytes_sent = (uint64_t *)calloc((size_t)p, 8);
    R->tmp = (float *)malloc((R->ce + 1) * sizeof(float));
    for (int r = 0; r < p; ++r) {
        R->work[r] = (float *)malloc((n + 1) * sizeof(float));
        memcpy(R->work[r], g_local[r], n * sizeof(float));
        R->wire[r].payload = malloc(orc_payload_bytes(mode, R->ce) + 1);
        R->wire[r].scales = (float *)malloc((orc_num_scales(mode, R->ce) + 1) * sizeof(float));
        R->res_payload[r] = calloc(orc_payload_bytes(mode, n) + 1, 1);
        R->res_scales[r] = (float *)calloc(orc_num_scales(mode, n) + 1, sizeof(float));
    }
    return R;
}

void orc_ring_free(orc_ring *R)
{
    if (!R) return;
    for (int r = 0; r < R->p; ++r) {
        free(R->work[r]); free(R->wire[r].payload); free(R->wire[r].scales);
        free(R->res_payload[r]); free(R->res_scales[r]);
    }
    free(R->work); free(R->wire); free(R->res_payload); free(R->res_scales);
    free(R->elems_sent); free(R->elems_reduced); free(R->bytes_sent); free(R->tmp);
    free(R);
}

/* Worker r puts block c of its working vector on the wire, compressed. */
static void ring_send(orc_ring *R, int r, int c)
{
    size_t lo = chunk_lo(R->n, R->ce, c), hi = chunk_hi(R->n, R->ce, c);
    orc_msg *m = &R->wire[r];
    m->chunk = c; m->len = hi - lo;
    orc_compress(R->mode, R->work[r] + lo, m->len, m->payload, m->scales);
    R->elems_sent[r] += m->len;
    R->bytes_sent[r] += orc_payload_bytes(R->mode, m->len) + 4 * orc_num_scales(R->mode, m->len);
}

/* Transmit-and-reduce round s (0 <= s <= p-2), all workers in parallel:
 * worker r sends block (r-s) mod p to worker r+1 and sum-reduces the block
 * (r-s-1) mod p it receives from worker r-1 into its own full-precision
 * copy of that block.  */
void orc_ring_reduce_scatter_step(orc_ring *R, int s)
{
    int p = R->p;
    for (int r = 0; r < p; ++r) ring_send(R, r, modp(r - s, p));
    for (int r = 0; r < p; ++r) {
        const orc_msg *m = &R->wire[modp(r - 1, p)];
        size_t lo = chunk_lo(R->n, R->ce, m->chunk);
        orc_decompress(R->mode, m->payload, m->scales, m->len, R->tmp);
        float *mine = R->work[r] + lo;
        for (size_t i = 0; i < m->len; ++i) mine[i] = R->tmp[i] + mine[i];
        R->elems_reduced[r] += m->len;
    }
    R->rounds += 1;
}

/* Which block worker r holds fully reduced once the p-1 rounds are over. */
int orc_ring_owner_chunk(const orc_ring *R, int r) { return modp(r + 1, R->p); }

/* The owner turns its fully reduced block into the compressed form that
 * travels round the ring, and keeps that same compressed form as its own
 * copy of the result, so that all replicas hold identical bytes. */
void orc_ring_seal(orc_ring *R)
{
    for (int r = 0; r < R->p; ++r) {
        int c = orc_ring_owner_chunk(R, r);
        size_t lo = chunk_lo(R->n, R->ce, c), hi = chunk_hi(R->n, R->ce, c);
        char *dst = (char *)R->res_payload[r] + orc_payload_bytes(R->mode, lo);
        orc_compress(R->mode, R->work[r] + lo, hi - lo, dst,
                     R->res_scales[r] + lo / ORC_QBLOCK);
    }
}

/* Send-back round s (0 <= s <= p-2): worker r forwards the compressed block
 * (r+1-s) mod p from its result slot; worker r+1 stores the bytes as they
 * arrive.  No arithmetic happens here. */
void orc_ring_allgather_step(orc_ring *R, int s)
{
    int p = R->p;
    for (int r = 0; r < p; ++r) {
        int c = modp(r + 1 - s, p);
        int to = modp(r + 1, p);
        size_t lo = chunk_lo(R->n, R->ce, c), hi = chunk_hi(R->n, R->ce, c);
        size_t len = hi - lo;
        size_t off = orc_payload_bytes(R->mode, lo), nb = orc_payload_bytes(R->mode, len);
        memcpy((char *)R->res_payload[to] + off, (const char *)R->res_payload[r] + off, nb);
        size_t ns = orc_num_scales(R->mode, len);
        if (ns) memcpy(R->res_scales[to] + lo / ORC_QBLOCK, R->res_scales[r] + lo / ORC_QBLOCK, ns * 4);
        R->elems_sent[r] += len;
        R->bytes_sent[r] += nb + 4 * ns;
    }
    R->rounds += 1;
}

const float *orc_ring_work(const orc_ring *R, int r) { return R->work[r]; }
const void  *orc_ring_result_payload(const orc_ring *R, int r) { return R->res_payload[r]; }
const float *orc_ring_result_scales(const orc_ring *R, int r) { return R->res_scales[r]; }
int      orc_ring_rounds(const orc_ring *R) { return R->rounds; }
uint64_t orc_ring_elems_sent(const orc_ring *R, int r) { return R->elems_sent[r]; }
uint64_t orc_ring_elems_reduced(const orc_ring *R, int r) { return R->elems_reduced[r]; }
uint64_t orc_ring_bytes_sent(const orc_ring *R, int r) { return R->bytes_sent[r]; }

/* AllReduce g^c_sum <- sum over workers of g_local (Alg. 1, communication
 * thread line 4), result left in compressed format on every worker. */
void orc_allreduce(int mode, int p, size_t n, const float *const *g_local,
                   void *const *out_payload, float *const *out_scales)
{
    orc_ring *R = orc_ring_new(mode, p, n, g_local);
    for (int s = 0; s + 1 < p; ++s) orc_ring_reduce_scatter_step(R, s);
    orc_ring_seal(R);
    for (int s = 0; s + 1 < p; ++s) orc_ring_allgather_step(R, s);
    for (int r = 0; r < p; ++r) {
        memcpy(out_payload[r], R->res_payload[r], orc_payload_bytes(mode, n));
        size_t ns = orc_num_scales(mode, n);
        if (ns) memcpy(out_scales[r], R->res_scales[r], ns * 4);
    }
    orc_ring_free(R);
}

/* ------------------------------------------------ direct (one-exchange) -- */

/* A second AllReduce schedule with the same definition of the result (Sec. 3.1
 * notes that its conclusions carry over to other AllReduce algorithms): every
 * worker is the owner of one block.  Exchange 1: worker k sends the compressed
 * block j of its gradient straight to owner j, for every j != k.  The owner
 * starts from its own full-precision block and adds the decompressed
 * contributions in the order of increasing ring distance (j+1, j+2, ...), then
 * compresses once.  Exchange 2: the owner sends the compressed result to everyone.
 * Two exchanges instead of 2(p-1) rounds, the same volume, and every value goes through
 * the codec twice instead of p times.  counters (may be NULL): [0] rounds,
 * [1] elements sent by worker 0, [2] elements reduced by worker 0. */
void orc_allreduce_direct(int mode, int p, size_t n, const float *const *g_local,
                          void *const *out_payload, float *const *out_scales, uint64_t *counters)
{
    size_t ce = orc_chunk_elems(n, p);
    float *P = (float *)malloc((ce + 1) * sizeof(float));
    float *tmp = (float *)malloc((ce + 1) * sizeof(float));
    void *msg = malloc(orc_payload_bytes(mode, ce) + 1);
    float *msg_sc = (float *)malloc((orc_num_scales(mode, ce) + 1) * sizeof(float));
    uint64_t sent0 = 0, reduced0 = 0;
    for (int j = 0; j < p; ++j) {                       /* owner j, block j */
        size_t lo = chunk_lo(n, ce, j), hi = chunk_hi(n, ce, j), len = hi - lo;
        for (size_t i = 0; i < len; ++i) P[i] = g_local[j][lo + i];
        for (int d = 1; d < p; ++d) {
            int k = modp(j + d, p);
            orc_compress(mode, g_local[k] + lo, len, msg, msg_sc);      /* exchange 1: k -> j */
            orc_decompress(mode, msg, msg_sc, len, tmp);
            for (size_t i = 0; i < len; ++i) P[i] = P[i] + tmp[i];
            if (k == 0) sent0 += len;
            if (j == 0) reduced0 += len;
        }
        orc_compress(mode, P, len, msg, msg_sc);
        for (int r = 0; r < p; ++r) {                   /* exchange 2: j -> everyone (and its own copy) */
            memcpy((char *)out_payload[r] + orc_payload_bytes(mode, lo), msg, orc_payload_bytes(mode, len));
            size_t ns = orc_num_scales(mode, len);
            if (ns) memcpy(out_scales[r] + lo / ORC_QBLOCK, msg_sc, ns * 4);
        }
        if (j == 0) sent0 += (uint64_t)(p - 1) * len;
    }
    if (counters) { counters[0] = p > 1 ? 2 : 0; counters[1] = sent0; counters[2] = reduced0; }
    free(P); free(tmp); free(msg); free(msg_sc);
}

/* ------------------------------------- recursive halving and doubling -- */

/* A third AllReduce schedule, one of those Sec. 3.1 names next to the ring
 * (recursive halving and doubling, after Thakur, Rabenseifner and Gropp,
 * 2005); p must be a power of two.  Blocks and the codec are the ring's.
 *
 * Reduce-scatter by recursive halving, rounds k = 0 .. log2(p)-1, distance
 * h = p / 2^(k+1): worker r and its partner r XOR h hold partial sums over the
 * same 2h consecutive blocks (the blocks whose index agrees with r above bit
 * h).  r keeps the h blocks whose index also agrees with r in bit h and sends
 * the other h, compressed, to the partner; the partner does the reverse.  Each
 * adds what it receives, decompressed, to its own full-precision partial sum
 * (the first round's "partial sum" is the local gradient).  After the last
 * round worker r holds block r fully reduced and compresses it once.
 *
 * All-gather by recursive doubling, distances d = 1, 2, .. p/2: worker r and
 * r XOR d swap, byte for byte, every compressed block they hold.
 *
 * For p = 4, block c:  P = (g_c + D(C(g_{c^2}))) + D(C(g_{c^1} + D(C(g_{c^3})))),
 * a codec chain of depth log2(p) instead of the ring's p-1.
 * counters (may be NULL): [0] rounds, [1] elements sent by worker 0,
 * [2] elements worker 0 received and added. */
int orc_allreduce_hd(int mode, int p, size_t n, const float *const *g_local,
                     void *const *out_payload, float *const *out_scales, uint64_t *counters)
{
    if (p < 1 || (p & (p - 1)) != 0) return -1;
    size_t ce = orc_chunk_elems(n, p);
    size_t pb = orc_payload_bytes(mode, n), ns = orc_num_scales(mode, n);
    float **acc = (float **)malloc((size_t)p * sizeof(*acc));           /* each worker's partial sums   */
    char **msg = (char **)malloc((size_t)p * sizeof(*msg));             /* what each worker sends       */
    float **msg_sc = (float **)malloc((size_t)p * sizeof(*msg_sc));
    float *tmp = (float *)malloc((n + 1) * sizeof(float));
    for (int r = 0; r < p; ++r) {
        acc[r] = (float *)malloc((n + 1) * sizeof(float));
        memcpy(acc[r], g_local[r], n * sizeof(float));
        msg[r] = (char *)malloc(pb + 1);
        msg_sc[r] = (float *)malloc((ns + 1) * sizeof(float));
    }
    uint64_t sent0 = 0, reduced0 = 0;
    int rounds = 0;

    for (int h = p / 2; h >= 1; h /= 2) {               /* halving rounds */
        for (int r = 0; r < p; ++r) {                   /* everyone sends ... */
            int keep0 = r & ~(h - 1), send0 = keep0 ^ h;
            size_t lo = chunk_lo(n, ce, send0), hi = chunk_hi(n, ce, send0 + h - 1);
            if (hi < lo) hi = lo;
            orc_compress(mode, acc[r] + lo, hi - lo, msg[r] + orc_payload_bytes(mode, lo), msg_sc[r] + lo / ORC_QBLOCK);
            if (r == 0) sent0 += hi - lo;
        }
        for (int r = 0; r < p; ++r) {                   /* ... then everyone receives and sums */
            int partner = r ^ h, keep0 = r & ~(h - 1);
            size_t lo = chunk_lo(n, ce, keep0), hi = chunk_hi(n, ce, keep0 + h - 1);
            if (hi < lo) hi = lo;
            orc_decompress(mode, msg[partner] + orc_payload_bytes(mode, lo), msg_sc[partner] + lo / ORC_QBLOCK, hi - lo, tmp);
            for (size_t i = 0; i < hi - lo; ++i) acc[r][lo + i] = acc[r][lo + i] + tmp[i];
            if (r == 0) reduced0 += hi - lo;
        }
        ++rounds;
    }

    for (int r = 0; r < p; ++r) {                       /* the owner compresses its block once */
        size_t lo = chunk_lo(n, ce, r), hi = chunk_hi(n, ce, r);
        orc_compress(mode, acc[r] + lo, hi - lo, (char *)out_payload[r] + orc_payload_bytes(mode, lo),
                     ns ? out_scales[r] + lo / ORC_QBLOCK : NULL);
    }
    for (int d = 1; d < p; d *= 2) {                    /* doubling rounds: r takes what r XOR d holds */
        for (int r = 0; r < p; ++r) {
            int partner = r ^ d, have0 = partner & ~(d - 1);
            size_t lo = chunk_lo(n, ce, have0), hi = chunk_hi(n, ce, have0 + d - 1);
            if (hi < lo) hi = lo;
            memcpy((char *)out_payload[r] + orc_payload_bytes(mode, lo),
                   (const char *)out_payload[partner] + orc_payload_bytes(mode, lo), orc_payload_bytes(mode, hi - lo));
            size_t k = orc_num_scales(mode, hi - lo);
            if (k) memcpy(out_scales[r] + lo / ORC_QBLOCK, out_scales[partner] + lo / ORC_QBLOCK, k * 4);
            if (partner == 0) sent0 += hi - lo;
        }
        ++rounds;
    }
    if (counters) { counters[0] = (uint64_t)rounds; counters[1] = sent0; counters[2] = reduced0; }
    for (int r = 0; r < p; ++r) { free(acc[r]); free(msg[r]); free(msg_sc[r]); }
    free(acc); free(msg); free(msg_sc); free(tmp);
    return 0;
}

/* --------------------------------------------------------------- update -- */

/* Alg. 1 compute thread, lines 4-5, for one model replica: decompress the
 * aggregated gradient handed in (the caller chooses which iteration's -- the
 * pipelined method hands in iteration t-K's, K = 2 in the optimal setting),
 * then step.  momentum == 0 is the paper's plain update; v is not touched. */
void orc_sgd_update(int mode, const void *g_sum_c, const float *scales, size_t n,
                    float *w, float *v, float lr, float momentum, float grad_scale)
{
    float *g = (float *)malloc((n + 1) * sizeof(float));
    orc_decompress(mode, g_sum_c, scales, n, g);
    for (size_t i = 0; i < n; ++i) {
        float gi = g[i];
        if (grad_scale != 1.0f) gi = gi * grad_scale;
        if (momentum != 0.0f) {
            v[i] = fmaf(momentum, v[i], gi);
            w[i] = fmaf(-lr, v[i], w[i]);
        } else {
            w[i] = fmaf(-lr, gi, w[i]);
        }
    }
    free(g);
}
