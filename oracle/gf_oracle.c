/*
 * CPU checker for the GradientFlow gradient-aggregation path (arxiv 1902.06855).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, literal statement of what
 * the path computes, used by tests, the smoke check and the CPU-baseline leg
 * of the benchmark.  It shares no code, header, table or helper with the HIP
 * library and the product never calls it.
 *
 * Every routine takes the steps in the order the paper states them, one
 * element at a time, with no blocking, fusion or reordering.  Floating-point
 * work on values that travel (accumulate, scale, casts, ring hops, unpack) is
 * done in the precision the method fixes (fp32 / fp16, round to nearest even,
 * subnormals kept); norms and scores are summed in fp64.
 *
 * Parity pins (tests/test_oracle_*.py): the two casts against numpy's float16;
 * layout against the closed form of Section 3.1; buckets against hand-worked
 * lists; the hop-by-hop ring against the rotated fold, against exact integer
 * sums and against the traffic formula of Section 2.4; the hierarchical
 * allreduce, message by message, against its formula, hand-worked fp16 sums
 * that tell the chain and rotation orders apart, exact integer sums and the
 * message size of Section 2.4; selection against a full sort (scores that are
 * not numbers included); pack, cast, unpack and the SGD update on both wire
 * types against numpy's fp32 / fp16 arithmetic element by element; residual
 * bookkeeping against the conservation property stated with Algorithm 1 on
 * both wire types; the warm-up chunk counts against hand-worked values.  The
 * same pins run once more against a build of this file under AddressSanitizer
 * and UndefinedBehaviorSanitizer.  Whole iterations (the paper prints no worked
 * example): against a job simulated worker by worker in plain Python, whose
 * workers meet only in the two exchanges of Section 3.2 and pass the packed
 * buffer hop by hop around the ring, on tiny sizes, every buffer bit for bit.
 *
 * The only parallelism is an OpenMP loop over workers (or over disjoint
 * element ranges of the ring), which changes no arithmetic and no order
 * within any sum.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- threads */

void gfo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int gfo_get_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------- fp32 <-> fp16 (Sec. 2.5)
 * Mixed precision sends IEEE binary16 gradients; the paper does not name a
 * rounding mode, so the IEEE default is taken: round to nearest, ties to
 * even, subnormal results kept, overflow to infinity. */

static uint32_t f32_bits(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
static float bits_f32(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }

uint16_t gfo_f32_to_f16(float x)
{
    uint32_t u = f32_bits(x);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    int32_t e = (int32_t)((u >> 23) & 0xffu);
    uint32_t frac = u & 0x7fffffu;

    if (e == 0xff) {                       /* infinity or NaN */
        if (frac == 0) return (uint16_t)(sign | 0x7c00u);
        return (uint16_t)(sign | 0x7e00u | (frac >> 13));   /* quiet NaN */
    }
    if (e == 0) return sign;               /* |x| < 2^-126: far below half's 2^-25 */

    int32_t E = e - 127;                   /* x = 1.frac * 2^E */
    if (E >= 16) return (uint16_t)(sign | 0x7c00u);
    if (E >= -14) {                        /* lands in half's normal range (before rounding) */
        uint32_t h = ((uint32_t)(E + 15) << 10) | (frac >> 13);
        uint32_t rem = frac & 0x1fffu;     /* 13 discarded bits */
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1;  /* carry may reach inf */
        return (uint16_t)(sign | h);
    }
    /* subnormal half: result = round(x / 2^-24), an integer in [0, 1024] */
    uint32_t sig = frac | 0x800000u;       /* x = sig * 2^(E-23) */
    int32_t shift = -E - 1;                /* x / 2^-24 = sig / 2^shift, shift >= 14 */
    if (shift >= 25) return sign;          /* below half of the smallest subnormal */
    uint32_t q = sig >> shift;
    uint32_t rem = sig & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (q & 1u))) q += 1;
    return (uint16_t)(sign | q);
}

float gfo_f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t frac = h & 0x3ffu;
    if (e == 0x1f) return bits_f32(sign | 0x7f800000u | (frac << 13));
    if (e == 0) {                          /* zero or subnormal: frac * 2^-24, exact in fp32 */
        float v = (float)frac * 0x1p-24f;
        return sign ? -v : v;
    }
    return bits_f32(sign | ((e + 112u) << 23) | (frac << 13));
}

void gfo_f32_to_f16_array(const float *x, uint16_t *h, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) h[i] = gfo_f32_to_f16(x[i]);
}

void gfo_f16_to_f32_array(const uint16_t *h, float *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = gfo_f16_to_f32(h[i]);
}

/* One ring hop on fp16 wire data: the partial sum is itself an fp16 message,
 * so the sum of two halves is rounded to half.  The fp32 sum of two halves is
 * rounded once to 24 bits and once more to 11; 24 >= 2*11+2 makes the second
 * rounding give the correctly rounded half sum. */
uint16_t gfo_f16_add(uint16_t a, uint16_t b)
{
    float s = gfo_f16_to_f32(a) + gfo_f16_to_f32(b);
    return gfo_f32_to_f16(s);
}

/* --------------------------------------------- memory pool layout (Sec. 3.1)
 * Tensors 1..m are given in ID order; backward produces tensor m first, so
 * tensor j occupies [ sum_{i>j} size_i , sum_{i>=j} size_i ). */
int64_t gfo_layout(const int64_t *size, int32_t m, int64_t *off)
{
    int64_t run = 0;
    for (int32_t j = m - 1; j >= 0; --j) { off[j] = run; run += size[j]; }
    return run;
}

/* ------------------------------------------------ lazy allreduce (Sec. 3.1)
 * Walk tensors in generation order (m down to 1); keep waiting while the
 * waited size is not greater than theta; once it is, the waited tensors form
 * one allreduce.  Whatever is still waiting after tensor 1 is flushed.
 * Returns the bucket count; bucket b covers pool range [lo[b], hi[b]). */
int32_t gfo_buckets(const int64_t *size, int32_t m, int64_t theta, int64_t *lo, int64_t *hi)
{
    int32_t nb = 0;
    int64_t start = 0, pos = 0, waited = 0;
    for (int32_t j = m - 1; j >= 0; --j) {
        pos += size[j];
        waited += size[j];
        if (waited > theta) {
            lo[nb] = start; hi[nb] = pos; ++nb;
            start = pos; waited = 0;
        }
    }
    if (waited > 0) { lo[nb] = start; hi[nb] = pos; ++nb; }
    return nb;
}

/* ----------------------------------------------------- chunks (Sec. 3.2)
 * The pool is cut into chunks of C gradients regardless of tensor borders;
 * the last one holds what is left. */
int64_t gfo_n_chunks(int64_t N, int64_t C) { return (N + C - 1) / C; }

static int64_t chunk_len(int64_t N, int64_t C, int64_t c)
{
    int64_t lo = c * C, hi = lo + C;
    if (hi > N) hi = N;
    return hi - lo;
}

/* Length of the packed buffer for an ascending selection. */
int64_t gfo_packed_len(int64_t N, int64_t C, const int32_t *sel, int32_t k)
{
    int64_t L = 0;
    for (int32_t j = 0; j < k; ++j) L += chunk_len(N, C, sel[j]);
    return L;
}

/* CSC relies on lazy allreduce as well (Sec. 3.2): important chunks are copied
 * to the buffer as they fill, in generation order, and an allreduce starts on
 * what is waiting once that is more than theta.  Returns the number of
 * buckets of the packed buffer; bucket b covers packed range [lo[b], hi[b]). */
int32_t gfo_packed_buckets(int64_t N, int64_t C, const int32_t *sel, int32_t k, int64_t theta,
                           int64_t *lo, int64_t *hi)
{
    int32_t nb = 0;
    int64_t start = 0, pos = 0, waited = 0;
    for (int32_t j = 0; j < k; ++j) {
        int64_t len = chunk_len(N, C, sel[j]);
        pos += len;
        waited += len;
        if (waited > theta) {
            lo[nb] = start; hi[nb] = pos; ++nb;
            start = pos; waited = 0;
        }
    }
    if (waited > 0) { lo[nb] = start; hi[nb] = pos; ++nb; }
    return nb;
}

/* Warm-up dense training (Sec. 3.2): start dense (zero sparsity ratio) and ramp
 * the sparsity ratio linearly to its final value over the warm-up iterations.
 * Returns how many chunks are important at 0-based iteration t. */
int64_t gfo_warmup_k(int64_t n_chunks, double final_density, int64_t t, int64_t warmup)
{
    double final_sparsity = 1.0 - final_density;
    double sparsity = final_sparsity;
    if (warmup > 0 && t < warmup) sparsity = final_sparsity * (double)t / (double)warmup;
    double density = 1.0 - sparsity;
    int64_t k = (int64_t)ceil(density * (double)n_chunks - 1e-9);
    if (k < 1) k = 1;
    if (k > n_chunks) k = n_chunks;
    return k;
}

/* ------------------------- Algorithm 1, allreduce preprocess: g = g + hg */
void gfo_accumulate(const float *g, const float *hg, float *acc, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) acc[i] = g[i] + hg[i];
}

/* -------------------------------------- per-chunk L1 norm (Sec. 3.2), fp64 */
void gfo_chunk_l1(const float *acc, int64_t N, int64_t C, double *l1)
{
    int64_t nc = gfo_n_chunks(N, C);
    for (int64_t c = 0; c < nc; ++c) {
        int64_t lo = c * C, len = chunk_len(N, C, c);
        double s = 0.0;
        for (int64_t i = 0; i < len; ++i) s += fabs((double)acc[lo + i]);
        l1[c] = s;
    }
}

/* Workers-major convenience: acc is [P][N], l1f is [P][nc] stored as fp32
 * (the norm vector that is exchanged holds single-precision values). */
void gfo_chunk_l1_workers(const float *acc, int32_t P, int64_t N, int64_t C, float *l1f)
{
    int64_t nc = gfo_n_chunks(N, C);
#pragma omp parallel for schedule(static)
    for (int32_t p = 0; p < P; ++p) {
        double *tmp = (double *)malloc((size_t)nc * sizeof(double));
        gfo_chunk_l1(acc + (int64_t)p * N, N, C, tmp);
        for (int64_t c = 0; c < nc; ++c) l1f[(int64_t)p * nc + c] = (float)tmp[c];
        free(tmp);
    }
}

/* ------------------------------------------ importance score (Sec. 3.2)
 * Every GPU holds one norm per chunk.  A chunk that went through this
 * iteration's allreduce holds the same (global) values everywhere, so each
 * GPU divides its norm by the number of GPUs before the norms are summed
 * across GPUs; any other chunk contributes its local norm.
 * l1f [P][nc]: local norms.  sent (ascending, k_sent entries) lists the chunks
 * reduced this iteration and red_l1[j] is the norm of the reduced values of
 * sent[j].  The score vector is single precision. */
void gfo_score(const float *l1f, int32_t P, int64_t nc,
               const int32_t *sent, int32_t k_sent, const float *red_l1, float *score)
{
    for (int64_t c = 0; c < nc; ++c) {
        double s = 0.0;
        for (int32_t p = 0; p < P; ++p) s += (double)l1f[(int64_t)p * nc + c];
        score[c] = (float)s;
    }
    for (int32_t j = 0; j < k_sent; ++j) {
        double s = 0.0;
        for (int32_t p = 0; p < P; ++p) s += (double)red_l1[j] / (double)P;
        score[sent[j]] = (float)s;
    }
}

/* ------------------------------------------------ top-k chunks (Sec. 3.2)
 * The k chunks with the largest score; equal scores go to the lower chunk
 * index; the answer is listed in ascending chunk order.  The paper does not
 * say what a chunk whose norm is not a number is worth; the reading taken is
 * that it ranks above every number (a worker whose gradients overflowed gets
 * them exchanged, as dense training would), all such chunks tying. */
typedef struct { float s; int32_t c; } gfo_key;

static int key_cmp(const void *a, const void *b)
{
    const gfo_key *x = (const gfo_key *)a, *y = (const gfo_key *)b;
    int xn = isnan(x->s), yn = isnan(y->s);
    if (xn != yn) return xn ? -1 : 1;
    if (!xn) {
        if (x->s > y->s) return -1;
        if (x->s < y->s) return 1;
    }
    return (x->c > y->c) - (x->c < y->c);
}

static int i32_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

void gfo_select(const float *score, int64_t nc, int32_t k, int32_t *sel, uint8_t *mask)
{
    gfo_key *keys = (gfo_key *)malloc((size_t)nc * sizeof(gfo_key));
    for (int64_t c = 0; c < nc; ++c) { keys[c].s = score[c]; keys[c].c = (int32_t)c; }
    qsort(keys, (size_t)nc, sizeof(gfo_key), key_cmp);
    for (int32_t j = 0; j < k; ++j) sel[j] = keys[j].c;
    qsort(sel, (size_t)k, sizeof(int32_t), i32_cmp);
    if (mask) {
        memset(mask, 0, (size_t)nc);
        for (int32_t j = 0; j < k; ++j) mask[sel[j]] = 1;
    }
    free(keys);
}

/* -------------------- pack + historical gradient (Sec. 3.2, Algorithm 1)
 * acc = g + hg has been formed.  Important chunks are copied, in ascending
 * chunk order, into the send buffer as fp16(acc * S) and their historical
 * gradient becomes 0; elsewhere hg = momentum * acc. */
void gfo_pack_residual(const float *acc, int64_t N, int64_t C,
                       const int32_t *sel, int32_t k, float S, float mu,
                       uint16_t *send, float *hg)
{
    int64_t nc = gfo_n_chunks(N, C);
    int64_t slot = 0;
    int32_t j = 0;
    for (int64_t c = 0; c < nc; ++c) {
        int64_t lo = c * C, len = chunk_len(N, C, c);
        if (j < k && sel[j] == c) {
            for (int64_t i = 0; i < len; ++i) {
                float scaled = acc[lo + i] * S;
                send[slot + i] = gfo_f32_to_f16(scaled);
                hg[lo + i] = 0.0f;
            }
            slot += len; ++j;
        } else {
            for (int64_t i = 0; i < len; ++i) hg[lo + i] = mu * acc[lo + i];
        }
    }
}

/* fp32 wire variant (the paper's single-precision baseline of Sec. 2.3). */
void gfo_pack_residual_f32(const float *acc, int64_t N, int64_t C,
                           const int32_t *sel, int32_t k, float S, float mu,
                           float *send, float *hg)
{
    int64_t nc = gfo_n_chunks(N, C);
    int64_t slot = 0;
    int32_t j = 0;
    for (int64_t c = 0; c < nc; ++c) {
        int64_t lo = c * C, len = chunk_len(N, C, c);
        if (j < k && sel[j] == c) {
            for (int64_t i = 0; i < len; ++i) { send[slot + i] = acc[lo + i] * S; hg[lo + i] = 0.0f; }
            slot += len; ++j;
        } else {
            for (int64_t i = 0; i < len; ++i) hg[lo + i] = mu * acc[lo + i];
        }
    }
}

/* Dense path: every gradient is cast, there is no historical gradient. */
void gfo_cast_dense(const float *g, int64_t n, float S, uint16_t *send)
{
    for (int64_t i = 0; i < n; ++i) { float scaled = g[i] * S; send[i] = gfo_f32_to_f16(scaled); }
}

void gfo_scale_dense_f32(const float *g, int64_t n, float S, float *send)
{
    for (int64_t i = 0; i < n; ++i) send[i] = g[i] * S;
}

/* --------------------------------------------- ring allreduce (Sec. 2.4)
 * wire: 0 = fp16 elements (2 bytes), 1 = fp32 elements (4 bytes).
 * The L elements are cut into P segments of seg = roundup(ceil(L/P), A)
 * elements, A = 16 bytes worth (8 halves / 4 floats); trailing segments may be
 * short or empty. */
static int64_t ring_seg(int64_t L, int32_t P, int wire)
{
    int64_t A = wire == 0 ? 8 : 4;
    int64_t s = (L + P - 1) / P;
    return (s + A - 1) / A * A;
}

int64_t gfo_ring_segment(int64_t L, int32_t P, int wire) { return ring_seg(L, P, wire); }

static void seg_range(int64_t L, int64_t seg, int64_t s, int64_t *lo, int64_t *hi)
{
    int64_t a = s * seg, b = a + seg;
    if (a > L) a = L;
    if (b > L) b = L;
    *lo = a; *hi = b;
}

static int imod(int a, int P) { int r = a % P; return r < 0 ? r + P : r; }

/* Message-passing emulation.  buf is [P][L] (rank-major), updated in place:
 * P-1 reduce-scatter steps, in each of which every rank r sends its segment
 * (r - t) mod P to rank r+1, which adds it to its own copy and rounds to the
 * wire type; then P-1 all-gather steps of plain copies.  sent[r] counts the
 * elements rank r put on the wire.  All messages of a step are taken before
 * any is applied (the ranks act at the same time). */
void gfo_ring_allreduce_hops(int wire, void *buf, int64_t L, int32_t P, int64_t *sent)
{
    size_t es = wire == 0 ? 2 : 4;
    int64_t seg = ring_seg(L, P, wire);
    unsigned char *base = (unsigned char *)buf;
    unsigned char *msg = (unsigned char *)malloc((size_t)P * (size_t)(seg ? seg : 1) * es);
    for (int32_t r = 0; r < P; ++r) sent[r] = 0;

    for (int phase = 0; phase < 2; ++phase) {
        for (int32_t t = 0; t < P - 1; ++t) {
            for (int32_t r = 0; r < P; ++r) {          /* every rank posts its message */
                int s = phase == 0 ? imod(r - t, P) : imod(r + 1 - t, P);
                int64_t lo, hi; seg_range(L, seg, s, &lo, &hi);
                memcpy(msg + (size_t)r * seg * es, base + ((size_t)r * L + lo) * es, (size_t)(hi - lo) * es);
                sent[r] += hi - lo;
            }
            for (int32_t r = 0; r < P; ++r) {          /* every rank's successor consumes it */
                int dst = imod(r + 1, P);
                int s = phase == 0 ? imod(r - t, P) : imod(r + 1 - t, P);
                int64_t lo, hi; seg_range(L, seg, s, &lo, &hi);
                if (phase == 1) {
                    memcpy(base + ((size_t)dst * L + lo) * es, msg + (size_t)r * seg * es, (size_t)(hi - lo) * es);
                } else if (wire == 0) {
                    const uint16_t *in = (const uint16_t *)(msg + (size_t)r * seg * es);
                    uint16_t *own = (uint16_t *)base + (size_t)dst * L + lo;
                    for (int64_t i = 0; i < hi - lo; ++i) own[i] = gfo_f16_add(in[i], own[i]);
                } else {
                    const float *in = (const float *)(msg + (size_t)r * seg * es);
                    float *own = (float *)base + (size_t)dst * L + lo;
                    for (int64_t i = 0; i < hi - lo; ++i) own[i] = in[i] + own[i];
                }
            }
        }
    }
    free(msg);
}

/* The same result written as what it is: element i of segment s is the left
 * fold x_s + x_{s+1} + ... + x_{s-1} (indices mod P), rounded to the wire type
 * after every addition.  x is [P][L], out is [L]. */
void gfo_ring_fold(int wire, const void *x, int64_t L, int32_t P, void *out)
{
    int64_t seg = ring_seg(L, P, wire);
#pragma omp parallel for schedule(static)
    for (int32_t s = 0; s < P; ++s) {
        int64_t lo, hi; seg_range(L, seg, s, &lo, &hi);
        for (int64_t i = lo; i < hi; ++i) {
            if (wire == 0) {
                const uint16_t *xs = (const uint16_t *)x;
                uint16_t v = xs[(size_t)s * L + i];
                for (int32_t j = 1; j < P; ++j) v = gfo_f16_add(v, xs[(size_t)imod(s + j, P) * L + i]);
                ((uint16_t *)out)[i] = v;
            } else {
                const float *xs = (const float *)x;
                float v = xs[(size_t)s * L + i];
                for (int32_t j = 1; j < P; ++j) v = v + xs[(size_t)imod(s + j, P) * L + i];
                ((float *)out)[i] = v;
            }
        }
    }
}

/* ------------------------------------ hierarchical allreduce (Sec. 2.4)
 * The P ranks form M groups of G = P / M consecutive ranks; the lowest rank of
 * a group is its master.  Three phases: a ring-based reduce inside each group
 * that leaves the group's sum on the master, a ring allreduce among the M
 * masters, a broadcast inside each group.
 *
 * Readings where the paper gives no detail: ranks send to their successor as
 * in the flat ring, so the reduce inside a group is a chain that starts at the
 * rank after the master and ends on the master (each rank adds its own values
 * to the partial sum it receives and rounds to the wire type); the broadcast is
 * the same chain run the other way round, plain copies.  The masters' ring
 * cuts the L elements into M segments (its message is L / M elements; the
 * L * M / P of the text is the same number in its 16-rank, 4-group example).
 *
 * Message-passing emulation, buf [P][L] updated in place; sent[r] counts the
 * elements rank r put on the wire over the three phases. */
void gfo_hier_allreduce_hops(int wire, void *buf, int64_t L, int32_t P, int32_t M, int64_t *sent)
{
    size_t es = wire == 0 ? 2 : 4;
    int32_t G = P / M;
    unsigned char *base = (unsigned char *)buf;
    for (int32_t r = 0; r < P; ++r) sent[r] = 0;

    /* phase 1: at step t the rank at local position 1 + t hands its partial sum on */
    for (int32_t t = 0; t + 1 < G; ++t) {
        for (int32_t g = 0; g < M; ++g) {
            int32_t src = g * G + 1 + t;
            int32_t dst = g * G + (2 + t) % G;
            sent[src] += L;
            if (wire == 0) {
                const uint16_t *in = (const uint16_t *)base + (size_t)src * L;
                uint16_t *own = (uint16_t *)base + (size_t)dst * L;
                for (int64_t i = 0; i < L; ++i) own[i] = gfo_f16_add(in[i], own[i]);
            } else {
                const float *in = (const float *)base + (size_t)src * L;
                float *own = (float *)base + (size_t)dst * L;
                for (int64_t i = 0; i < L; ++i) own[i] = in[i] + own[i];
            }
        }
    }

    /* phase 2: the flat ring among the masters */
    unsigned char *mast = (unsigned char *)malloc((size_t)M * (size_t)(L ? L : 1) * es);
    int64_t *msent = (int64_t *)malloc((size_t)M * sizeof(int64_t));
    for (int32_t g = 0; g < M; ++g) memcpy(mast + (size_t)g * L * es, base + (size_t)g * G * L * es, (size_t)L * es);
    gfo_ring_allreduce_hops(wire, mast, L, M, msent);
    for (int32_t g = 0; g < M; ++g) {
        memcpy(base + (size_t)g * G * L * es, mast + (size_t)g * L * es, (size_t)L * es);
        sent[g * G] += msent[g];
    }
    free(mast);
    free(msent);

    /* phase 3: master -> local 1 -> ... -> local G - 1 */
    for (int32_t t = 0; t + 1 < G; ++t) {
        for (int32_t g = 0; g < M; ++g) {
            int32_t src = g * G + t, dst = g * G + t + 1;
            sent[src] += L;
            memcpy(base + (size_t)dst * L * es, base + (size_t)src * L * es, (size_t)L * es);
        }
    }
}

/* The same result as a formula: y_g = x_{gG+1} + x_{gG+2} + ... + x_{gG+G-1} + x_{gG}
 * (left to right), and element i of the masters' segment s is the left fold
 * y_s + y_{s+1} + ... + y_{s-1} (indices mod M); every addition rounds to the
 * wire type.  x is [P][L], out is [L]. */
void gfo_hier_fold(int wire, const void *x, int64_t L, int32_t P, int32_t M, void *out)
{
    int32_t G = P / M;
    int64_t seg = ring_seg(L, M, wire);
#pragma omp parallel for schedule(static)
    for (int32_t s = 0; s < M; ++s) {
        int64_t lo, hi; seg_range(L, seg, s, &lo, &hi);
        for (int64_t i = lo; i < hi; ++i) {
            if (wire == 0) {
                const uint16_t *xs = (const uint16_t *)x;
                uint16_t v = 0;
                for (int32_t j = 0; j < M; ++j) {
                    int32_t g = imod(s + j, M);
                    uint16_t y = xs[(size_t)(g * G + 1 % G) * L + i];
                    for (int32_t q = 2; q <= G; ++q) y = gfo_f16_add(y, xs[(size_t)(g * G + q % G) * L + i]);
                    v = j == 0 ? y : gfo_f16_add(v, y);
                }
                ((uint16_t *)out)[i] = v;
            } else {
                const float *xs = (const float *)x;
                float v = 0.0f;
                for (int32_t j = 0; j < M; ++j) {
                    int32_t g = imod(s + j, M);
                    float y = xs[(size_t)(g * G + 1 % G) * L + i];
                    for (int32_t q = 2; q <= G; ++q) y = y + xs[(size_t)(g * G + q % G) * L + i];
                    v = j == 0 ? y : v + y;
                }
                ((float *)out)[i] = v;
            }
        }
    }
}

/* --------------------------------- unpack (Sec. 2.5 second cast, Sec. 3.2)
 * Reduced wire values go back to fp32, times alpha (1 / loss scale), into the
 * positions of the important chunks only; everything else in `out` is left
 * alone.  red_l1[j] (optional) = L1 norm of what was written for sel[j],
 * summed in fp64 and stored in single precision. */
void gfo_unpack(int wire, const void *reduced, int64_t N, int64_t C,
                const int32_t *sel, int32_t k, float alpha, float *out, float *red_l1)
{
    int64_t slot = 0;
    for (int32_t j = 0; j < k; ++j) {
        int64_t lo = (int64_t)sel[j] * C, len = chunk_len(N, C, sel[j]);
        double s = 0.0;
        for (int64_t i = 0; i < len; ++i) {
            float v = wire == 0 ? gfo_f16_to_f32(((const uint16_t *)reduced)[slot + i])
                                : ((const float *)reduced)[slot + i];
            v = v * alpha;
            out[lo + i] = v;
            s += fabs((double)v);
        }
        if (red_l1) red_l1[j] = (float)s;
        slot += len;
    }
}

/* ------------------------------ Algorithm 1, SGD update step (Sec. 3.2)
 * For a gradient in an important chunk: u = hu = momentum * hu + learningrate * g
 * and w = w + u.  Anywhere else hu keeps its value and w is not updated.
 * g is the unpacked reduced gradient; out (optional) receives it.
 * Mixed precision (Sec. 2.5): the update works on FP32 values, forward and
 * backward on FP16 parameters; w_half (optional) is that FP16 copy, rewritten
 * from the new FP32 weight wherever a weight changed (one conversion each). */
void gfo_sgd_update(int wire, const void *reduced, int64_t N, int64_t C,
                    const int32_t *sel, int32_t k, float alpha, float momentum, float lr,
                    float *w, float *hu, float *out, uint16_t *w_half)
{
    int64_t slot = 0;
    for (int32_t j = 0; j < k; ++j) {
        int64_t lo = (int64_t)sel[j] * C, len = chunk_len(N, C, sel[j]);
        for (int64_t i = 0; i < len; ++i) {
            float g = wire == 0 ? gfo_f16_to_f32(((const uint16_t *)reduced)[slot + i])
                                : ((const float *)reduced)[slot + i];
            g = g * alpha;
            if (out) out[lo + i] = g;
            float keep = momentum * hu[lo + i];
            float step = lr * g;
            float u = keep + step;
            hu[lo + i] = u;
            w[lo + i] = w[lo + i] + u;
            if (w_half) w_half[lo + i] = gfo_f32_to_f16(w[lo + i]);
        }
        slot += len;
    }
}

void gfo_unpack_dense(int wire, const void *reduced, int64_t n, float alpha, float *out)
{
    for (int64_t i = 0; i < n; ++i) {
        float v = wire == 0 ? gfo_f16_to_f32(((const uint16_t *)reduced)[i])
                            : ((const float *)reduced)[i];
        out[i] = v * alpha;
    }
}

/* ---------------- worker-major batch forms (the same loops, once per worker) */

void gfo_accumulate_workers(const float *g, const float *hg, float *acc, int32_t P, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int32_t p = 0; p < P; ++p)
        gfo_accumulate(g + (int64_t)p * N, hg + (int64_t)p * N, acc + (int64_t)p * N, N);
}

void gfo_pack_residual_workers(int wire, const float *acc, int32_t P, int64_t N, int64_t C,
                               const int32_t *sel, int32_t k, float S, float mu,
                               void *send /* [P][L] */, float *hg /* [P][N] */)
{
    int64_t L = gfo_packed_len(N, C, sel, k);
#pragma omp parallel for schedule(static)
    for (int32_t p = 0; p < P; ++p) {
        if (wire == 0)
            gfo_pack_residual(acc + (int64_t)p * N, N, C, sel, k, S, mu,
                              (uint16_t *)send + (int64_t)p * L, hg + (int64_t)p * N);
        else
            gfo_pack_residual_f32(acc + (int64_t)p * N, N, C, sel, k, S, mu,
                                  (float *)send + (int64_t)p * L, hg + (int64_t)p * N);
    }
}

void gfo_cast_dense_workers(int wire, const float *g, int32_t P, int64_t N, float S, void *send)
{
#pragma omp parallel for schedule(static)
    for (int32_t p = 0; p < P; ++p) {
        if (wire == 0) gfo_cast_dense(g + (int64_t)p * N, N, S, (uint16_t *)send + (int64_t)p * N);
        else gfo_scale_dense_f32(g + (int64_t)p * N, N, S, (float *)send + (int64_t)p * N);
    }
}
