/*
 * CPU oracle for the MoSKA decode-attention path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, fp64 throughout, two-pass softmax, one row at a time: the un-batched
 * per-request formulation the paper starts from (Sec. I, Sec. III-A: a series of
 * GEMVs).  Nothing here is blocked, fused or reordered, and nothing is shared with
 * the GPU library.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it.
 *
 * Steps (notation: B requests, Hq query heads, Hkv KV heads, G = Hq/Hkv, head dim D,
 * C shared chunks of L tokens, top-k = k, U unique tokens, P = k+1 partial slots):
 *
 *   S1 scores   s[b,h,c] = (sum_{g<G} q[b,hG+g,:]) . E[h,c,:]      Sec. III-B: relevance =
 *                                                                   inner product of query and
 *                                                                   precomputed chunk embedding
 *   S2 select   ids[b,h,0..k-1] = first k chunks in the order       Sec. III-B: top-k subset
 *               (score descending, chunk id ascending)
 *   S3 direct   softmax attention of row (b,hq) over the union of    Fig. 2(b): the complete
 *               its k routed chunks and its own unique context       system's output
 *   S4 partial  the same attention restricted to one routed chunk    Sec. III-A: shared vs
 *               (slot j<k) or to the unique context (slot k),        unique attention
 *               reported as (O_p, LSE_p)
 *   S5 merge    log-sum-exp weighted combination of the partials    (implied by Fig. 2(b))
 *
 * Extension (not in the paper): T = q_len query tokens per request.  Query token (b,t) is row
 * b*T + t wherever the single-token path has row b; it is routed and attends to its shared chunks
 * on its own, and sees the first unique_len[b] - (T-1-t) tokens of the request's unique context
 * (the T new tokens are the last T of it: causal among themselves).  T = 1 is the paper's path.
 *
 * Readings where the paper is silent: the G heads of a group share one selection
 * and their scores add; routing uses q unscaled; LSE is the natural log of the sum
 * of exp(scale * q.k); an empty key set yields O = 0, LSE = -inf; no mask (decode).
 * Storage dtypes are widened exactly to fp64: f32, bf16, and OCP fp8 e4m3fn with a
 * per-(chunk, KV head) f32 scale, x = scale * decode(byte).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { MO_F32 = 0, MO_BF16 = 1, MO_FP8_E4M3 = 2, MO_F64 = 3 /* mo_attend only */ };

typedef struct {
    int32_t B, Hq, Hkv, D, C, L, k, U;
    int32_t q_dtype, kv_dtype;
    double scale;
    int32_t T;              /* query tokens per request, >= 1 */
} mo_problem;

static int64_t query_tokens(const mo_problem *p) { return (int64_t)p->B * (p->T > 0 ? p->T : 1); }

/* ---- exact widening of stored values ------------------------------------------------ */

static double widen_bf16(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* OCP 8-bit float e4m3fn: 1 sign, 4 exponent (bias 7), 3 mantissa; no infinities,
 * S.1111.111 is NaN, exponent 0 is subnormal m/8 * 2^-6. */
static double widen_fp8_e4m3fn(uint8_t b) {
    int s = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

static double load_as_f64(int dtype, const void *p, int64_t i) {
    switch (dtype) {
    case MO_F32: return (double)((const float *)p)[i];
    case MO_BF16: return widen_bf16(((const uint16_t *)p)[i]);
    case MO_FP8_E4M3: return widen_fp8_e4m3fn(((const uint8_t *)p)[i]);
    case MO_F64: return ((const double *)p)[i];
    default: return NAN;
    }
}

int mo_widen(int dtype, const void *src, int64_t n, double *dst) {
    if (dtype < 0 || dtype > 2) return -1;
    for (int64_t i = 0; i < n; ++i) dst[i] = load_as_f64(dtype, src, i);
    return 0;
}

int mo_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- S1 + S2: routing ---------------------------------------------------------------- */

typedef struct { double s; int32_t c; } scored;

static int by_score_desc_then_id(const void *a, const void *b) {
    const scored *x = a, *y = b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->c > y->c) - (x->c < y->c);
}

/* ids [B*T,Hkv,k]; sel_scores [B*T,Hkv,k] and all_scores [B*T,Hkv,C] may be NULL. */
int mo_route(const mo_problem *p, const void *Q, const void *E,
             int32_t *ids, double *sel_scores, double *all_scores) {
    if (p->k < 1 || p->k > p->C || p->Hq % p->Hkv) return -1;
    const int G = p->Hq / p->Hkv, D = p->D, C = p->C;
    int64_t rows = query_tokens(p) * p->Hkv;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / p->Hkv;                 /* query token */
        int h = (int)(r % p->Hkv);
        double *qs = malloc(sizeof(double) * D);
        scored *sc = malloc(sizeof(scored) * C);
        for (int d = 0; d < D; ++d) {
            double a = 0.0;
            for (int g = 0; g < G; ++g)
                a += load_as_f64(p->q_dtype, Q, (b * p->Hq + h * G + g) * D + d);
            qs[d] = a;
        }
        for (int c = 0; c < C; ++c) {
            double a = 0.0;
            for (int d = 0; d < D; ++d)
                a += qs[d] * load_as_f64(p->q_dtype, E, ((int64_t)h * C + c) * D + d);
            sc[c].s = a;
            sc[c].c = c;
            if (all_scores) all_scores[r * C + c] = a;
        }
        qsort(sc, C, sizeof(scored), by_score_desc_then_id);
        for (int j = 0; j < p->k; ++j) {
            ids[r * p->k + j] = sc[j].c;
            if (sel_scores) sel_scores[r * p->k + j] = sc[j].s;
        }
        free(qs);
        free(sc);
    }
    return 0;
}

/* ---- query aggregation (Sec. III-A): group routed items by (KV head, chunk) ---------- */

/* Item (b,h,j), b a query token, has index b*k+j inside head h and belongs to bucket h*C + ids[b,h,j].
 * off [Hkv*C+1] is the exclusive prefix sum of bucket sizes; items [B*Hkv*k] lists each
 * bucket's item indices in ascending order. */
int mo_bucket(const mo_problem *p, const int32_t *ids, int32_t *off, int32_t *items) {
    const int nb = p->Hkv * p->C;
    int32_t *fill = calloc(nb + 1, sizeof(int32_t));
    const int64_t nq = query_tokens(p);
    for (int i = 0; i <= nb; ++i) off[i] = 0;
    for (int64_t b = 0; b < nq; ++b)
        for (int h = 0; h < p->Hkv; ++h)
            for (int j = 0; j < p->k; ++j) {
                int c = ids[(b * p->Hkv + h) * p->k + j];
                if (c < 0 || c >= p->C) { free(fill); return -1; }
                off[h * p->C + c + 1] += 1;
            }
    for (int i = 0; i < nb; ++i) off[i + 1] += off[i];
    for (int64_t b = 0; b < nq; ++b)
        for (int h = 0; h < p->Hkv; ++h)
            for (int j = 0; j < p->k; ++j) {
                int bk = h * p->C + ids[(b * p->Hkv + h) * p->k + j];
                items[off[bk] + fill[bk]++] = (int32_t)(b * p->k + j);
            }
    free(fill);
    return 0;
}

/* ---- softmax attention of one query row over a list of key segments ------------------ */

typedef struct {
    int dtype;
    const void *K, *V;     /* n x D each, row-major, at element offset `base` */
    int64_t base;
    int64_t n;
    double kmul, vmul;     /* dequantisation scales (1 for f32/bf16) */
} segment;

/* O[D], *lse: attention of q over the concatenation of the segments.
 * Two passes: all logits and their maximum first, then exponentials. */
static void attend_segments(int D, const double *q, double scale,
                            const segment *seg, int nseg, double *O, double *lse) {
    int64_t n = 0;
    for (int s = 0; s < nseg; ++s) n += seg[s].n;
    for (int d = 0; d < D; ++d) O[d] = 0.0;
    if (n == 0) { *lse = -INFINITY; return; }
    double *z = malloc(sizeof(double) * n);
    double zmax = -INFINITY;
    int64_t t = 0;
    for (int s = 0; s < nseg; ++s)
        for (int64_t i = 0; i < seg[s].n; ++i, ++t) {
            double a = 0.0;
            for (int d = 0; d < D; ++d)
                a += q[d] * (seg[s].kmul * load_as_f64(seg[s].dtype, seg[s].K, seg[s].base + i * D + d));
            z[t] = scale * a;
            if (z[t] > zmax) zmax = z[t];
        }
    double denom = 0.0;
    t = 0;
    for (int s = 0; s < nseg; ++s)
        for (int64_t i = 0; i < seg[s].n; ++i, ++t) {
            double w = exp(z[t] - zmax);
            denom += w;
            for (int d = 0; d < D; ++d)
                O[d] += w * (seg[s].vmul * load_as_f64(seg[s].dtype, seg[s].V, seg[s].base + i * D + d));
        }
    for (int d = 0; d < D; ++d) O[d] /= denom;
    *lse = zmax + log(denom);
    free(z);
}

/* Exposed for tests: one row over one fp64 key set (K, V are n x D). */
int mo_attend(int D, int64_t n, const double *q, const double *K, const double *V,
              double scale, double *O, double *lse) {
    segment s = { MO_F64, K, V, 0, n, 1.0, 1.0 };
    attend_segments(D, q, scale, &s, 1, O, lse);
    return 0;
}

static segment shared_segment(const mo_problem *p, const void *Ks, const void *Vs,
                              const float *scale_k, const float *scale_v, int c, int h) {
    segment s;
    s.dtype = p->kv_dtype;
    s.K = Ks;
    s.V = Vs;
    s.base = ((int64_t)c * p->Hkv + h) * p->L * p->D;
    s.n = p->L;
    s.kmul = scale_k ? (double)scale_k[c * p->Hkv + h] : 1.0;
    s.vmul = scale_v ? (double)scale_v[c * p->Hkv + h] : 1.0;
    return s;
}

/* The unique context query token bq = b*T + t may see: the request's first len - (T-1-t) tokens. */
static segment unique_segment(const mo_problem *p, const void *Ku, const void *Vu,
                              const int32_t *unique_len, int64_t bq, int h) {
    const int T = p->T > 0 ? p->T : 1;
    const int64_t b = bq / T;
    const int t = (int)(bq % T);
    segment s;
    s.dtype = p->q_dtype;
    s.K = Ku;
    s.V = Vu;
    s.base = (b * p->Hkv + h) * p->U * p->D;
    s.n = (unique_len ? unique_len[b] : p->U) - (T - 1 - t);
    if (s.n < 0) s.n = 0;
    s.kmul = s.vmul = 1.0;
    return s;
}

/* ---- S4: partial attentions ----------------------------------------------------------- */

/* part_O [B*T,Hq,k+1,D], part_LSE [B*T,Hq,k+1]: slot j<k = chunk ids[b,h,j], slot k = unique. */
int mo_partials(const mo_problem *p, const void *Q, const void *Ks, const void *Vs,
                const float *scale_k, const float *scale_v, const void *Ku, const void *Vu,
                const int32_t *unique_len, const int32_t *ids, double *part_O, double *part_LSE) {
    const int G = p->Hq / p->Hkv, D = p->D, P = p->k + 1;
    int64_t rows = query_tokens(p) * p->Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / p->Hq;                  /* query token */
        int hq = (int)(r % p->Hq), h = hq / G;
        double *q = malloc(sizeof(double) * D);
        for (int d = 0; d < D; ++d) q[d] = load_as_f64(p->q_dtype, Q, r * D + d);
        for (int j = 0; j < P; ++j) {
            segment s = j < p->k
                ? shared_segment(p, Ks, Vs, scale_k, scale_v, ids[(b * p->Hkv + h) * p->k + j], h)
                : unique_segment(p, Ku, Vu, unique_len, b, h);
            attend_segments(D, q, p->scale, &s, 1, part_O + (r * P + j) * D, part_LSE + r * P + j);
        }
        free(q);
    }
    return 0;
}

/* ---- S3: direct result over the union ------------------------------------------------ */

int mo_direct(const mo_problem *p, const void *Q, const void *Ks, const void *Vs,
              const float *scale_k, const float *scale_v, const void *Ku, const void *Vu,
              const int32_t *unique_len, const int32_t *ids, double *O, double *LSE) {
    const int G = p->Hq / p->Hkv, D = p->D;
    int64_t rows = query_tokens(p) * p->Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        int64_t b = r / p->Hq;                  /* query token */
        int hq = (int)(r % p->Hq), h = hq / G;
        double *q = malloc(sizeof(double) * D);
        segment *seg = malloc(sizeof(segment) * (p->k + 1));
        for (int d = 0; d < D; ++d) q[d] = load_as_f64(p->q_dtype, Q, r * D + d);
        for (int j = 0; j < p->k; ++j)
            seg[j] = shared_segment(p, Ks, Vs, scale_k, scale_v, ids[(b * p->Hkv + h) * p->k + j], h);
        seg[p->k] = unique_segment(p, Ku, Vu, unique_len, b, h);
        attend_segments(D, q, p->scale, seg, p->k + 1, O + r * D, LSE + r);
        free(q);
        free(seg);
    }
    return 0;
}

/* ---- S5: log-sum-exp merge of partials ------------------------------------------------ */

/* For each of `rows` rows: m = max_p LSE_p, w_p = exp(LSE_p - m),
 * O = sum_p w_p O_p / sum_p w_p, LSE = m + ln sum_p w_p.  Slots with LSE = -inf weigh 0;
 * if every slot is empty the row is O = 0, LSE = -inf. */
int mo_merge(int64_t rows, int P, int D, const double *part_O, const double *part_LSE,
             double *O, double *LSE) {
    for (int64_t r = 0; r < rows; ++r) {
        double m = -INFINITY;
        for (int j = 0; j < P; ++j)
            if (part_LSE[r * P + j] > m) m = part_LSE[r * P + j];
        for (int d = 0; d < D; ++d) O[r * D + d] = 0.0;
        if (m == -INFINITY) { LSE[r] = -INFINITY; continue; }
        double wsum = 0.0;
        for (int j = 0; j < P; ++j) {
            double l = part_LSE[r * P + j];
            if (l == -INFINITY) continue;
            double w = exp(l - m);
            wsum += w;
            for (int d = 0; d < D; ++d) O[r * D + d] += w * part_O[(r * P + j) * D + d];
        }
        for (int d = 0; d < D; ++d) O[r * D + d] /= wsum;
        LSE[r] = m + log(wsum);
    }
    return 0;
}

/* ---- offline construction of the shared store (Sec. III-A/B: pre-computed caches and
 *      precomputed chunk embeddings) --------------------------------------------------------- */

/* round-to-nearest-even f64 -> bf16 bits via f32 (the value is first rounded to f32, as a GPU
 * kernel that accumulates in f64 and stores through f32 does) */
static uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* E[h,c,:] = mean over the L tokens of the stored keys of chunk c on KV head h (dequantised
 * when the store is fp8), accumulated in fp64, rounded to the q dtype (f32 or bf16). */
int mo_chunk_embeddings(const mo_problem *p, const void *Ks, const float *scale_k, void *E) {
    if (p->q_dtype != MO_F32 && p->q_dtype != MO_BF16) return -1;
    for (int c = 0; c < p->C; ++c)
        for (int h = 0; h < p->Hkv; ++h) {
            const double mul = scale_k ? (double)scale_k[c * p->Hkv + h] : 1.0;
            const int64_t base = ((int64_t)c * p->Hkv + h) * p->L * p->D;
            for (int d = 0; d < p->D; ++d) {
                double a = 0.0;
                for (int t = 0; t < p->L; ++t) a += load_as_f64(p->kv_dtype, Ks, base + (int64_t)t * p->D + d);
                const float m = (float)(mul * a / (double)p->L);
                const int64_t o = ((int64_t)h * p->C + c) * p->D + d;
                if (p->q_dtype == MO_F32) ((float *)E)[o] = m;
                else ((uint16_t *)E)[o] = f32_to_bf16_rne(m);
            }
        }
    return 0;
}

/* f32 -> OCP e4m3fn, round to nearest even, saturating at +-448 (inputs are finite) */
static uint8_t f32_to_fp8_e4m3fn_sat(float f) {
    uint8_t s = f < 0 || (f == 0 && signbit(f)) ? 0x80 : 0;
    double a = fabs((double)f);
    if (a >= 448.0) return s | 0x7E;
    if (a < ldexp(1.0, -10)) return s;                     /* below half the smallest subnormal (2^-9): zero;
                                                              exactly 2^-10 ties to even = 0 */
    int e;
    (void)frexp(a, &e);                                    /* a = m * 2^e, m in [0.5,1) -> exponent e-1 */
    int ex = e - 1;
    if (ex < -6) ex = -6;                                  /* subnormal range shares the exponent -6 */
    double q = ldexp(a, 3 - ex);                           /* units of the last mantissa bit */
    double r = nearbyint(q);                               /* default rounding mode: to nearest even */
    if (ex == -6 && r < 8) return s | (uint8_t)r;          /* subnormal (or rounds up to the first normal below) */
    if (r >= 16) { r = 8; ex += 1; }                       /* mantissa overflow */
    if (ex > 8 || (ex == 8 && r > 14)) return s | 0x7E;
    return s | (uint8_t)(((ex + 7) << 3) | ((int)r - 8));
}

/* Per (chunk, KV head): scale = amax/448 (f32 division), y = x/scale (f32 division), stored as
 * e4m3fn.  X [C,Hkv,L,D] in the q dtype (f32 or bf16).  An all-zero block gets scale 1e-30. */
int mo_quantize_fp8(const mo_problem *p, const void *X, uint8_t *X8, float *scale) {
    for (int c = 0; c < p->C; ++c)
        for (int h = 0; h < p->Hkv; ++h) {
            const int64_t base = ((int64_t)c * p->Hkv + h) * p->L * p->D, n = (int64_t)p->L * p->D;
            float amax = 0.f;
            for (int64_t i = 0; i < n; ++i) {
                float v = fabsf((float)load_as_f64(p->q_dtype, X, base + i));
                if (v > amax) amax = v;
            }
            float sc = amax / 448.0f;
            if (sc < 1e-30f) sc = 1e-30f;
            scale[c * p->Hkv + h] = sc;
            for (int64_t i = 0; i < n; ++i) {
                float y = (float)load_as_f64(p->q_dtype, X, base + i) / sc;
                X8[base + i] = f32_to_fp8_e4m3fn_sat(y);
            }
        }
    return 0;
}
