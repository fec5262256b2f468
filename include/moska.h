/*
 * moska.h -- C interface of the MI355X (gfx950) MoSKA decode-attention library.
 *
 * One decode step of one attention layer, for B concurrent requests with one query
 * token each (paper Sec. III, Fig. 2):
 *
 *   moska_route        score every shared KV chunk against each query group and keep the
 *                      top-k chunks per (request, KV head)                   (Sec. III-B)
 *   moska_bucket       group the routed (request, KV head, slot) items by chunk, so that
 *                      all queries aimed at one chunk form one query matrix  (Sec. III-A)
 *   moska_shared_attn  Shared KV Attention: one batched GEMM-shaped attention per
 *                      (chunk, KV head) bucket, emitting partial (O, LSE)    (Sec. III-A)
 *   moska_unique_attn  per-request attention over the request's own KV       (Sec. III-A)
 *   moska_merge        log-sum-exp combination of the k shared partials and the unique
 *                      partial into the layer's attention output             (Fig. 2(b))
 *
 * Notation: Hq query heads, Hkv KV heads, G = Hq/Hkv (query head hq reads KV head hq/G),
 * head dimension D, C shared chunks of L tokens each, top-k = k, U_max unique tokens per
 * request (request b uses the first unique_len[b]), P = k+1 partial slots per query row.
 *
 * Several query tokens per request (q_len = T > 1; an extension beyond the paper, for speculative
 * decoding or chunked prefill against the shared store): query token (b,t) takes the place of
 * request b in every shape below -- read B as B*T with row b*T + t -- except in Ku, Vu and
 * unique_len, which stay per request.  Each token is routed on its own and attends to all of its
 * routed chunks; the T tokens are the last T of the request's unique_len[b] unique tokens, and
 * token t attends to the first unique_len[b] - (T-1-t) of them (at least 0).
 *
 * Conventions common to every call
 *   - `p` and `out` are HOST pointers.  Every other pointer is a DEVICE pointer owned by
 *     the caller, 16-byte aligned, dense row-major in the stated shape (last index
 *     contiguous).  The library never allocates, frees or synchronises: all work is
 *     enqueued on `stream` (a hipStream_t passed as void*, NULL = the null stream).
 *   - Returns MOSKA_OK (0) or a negative moska_status_t.  Arguments are validated on the
 *     host before anything is launched: a failing call enqueues nothing.
 *   - The same buffers may be reused by later calls on the same stream; calls on
 *     different streams must not share output or workspace buffers.
 *   - Logits are scale * (q . k); LSE is the natural log of the sum of their
 *     exponentials; an empty key set gives O = 0, LSE = -inf.  No mask is applied: a
 *     decode query sees every token of every selected chunk and of its unique context.
 *   - Accumulation is fp32 (fp64 for routing scores).  With q_dtype = MOSKA_F32 all
 *     arithmetic is fp32 on the vector ALUs; with MOSKA_BF16 and D = 128 the two
 *     attention calls run on bf16 MFMA with fp32 accumulation (an FP8 store's scores on
 *     the scaled fp8 MFMA, the query carried as a pair of e4m3 values: bf16 precision).
 */
#ifndef MOSKA_H
#define MOSKA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOSKA_F32 = 0,
    MOSKA_BF16 = 1,
    MOSKA_FP8_E4M3 = 2      /* OCP e4m3fn: bias 7, max 448, no infinities */
} moska_dtype_t;

typedef enum {
    MOSKA_OK = 0,
    MOSKA_ERR_INVALID_ARG = -1,          /* null pointer, non-positive size, k > C, Hq % Hkv != 0 ... */
    MOSKA_ERR_UNSUPPORTED = -2,          /* dtype combination or size outside the built kernels */
    MOSKA_ERR_WORKSPACE_TOO_SMALL = -3,
    MOSKA_ERR_HIP = -4,                  /* a HIP runtime call (launch, attribute) failed */
    MOSKA_ERR_SCRATCH_LIMIT = -5         /* moska_decode_step_static: workspace need exceeds MOSKA_STATIC_SCRATCH_BYTES */
} moska_status_t;

typedef struct {
    int32_t B, Hq, Hkv, D;      /* D: multiple of 16, <= 256 */
    int32_t C, L, k;            /* shared store: C chunks x L tokens; 1 <= k <= C */
    int32_t U_max;              /* padded unique length, >= 0 */
    int32_t q_dtype;            /* MOSKA_F32 or MOSKA_BF16: dtype of Q, E, unique K/V and O */
    int32_t shared_kv_dtype;    /* MOSKA_F32 (only with q F32), MOSKA_BF16 or MOSKA_FP8_E4M3 (with q BF16) */
    float scale;                /* logit scale, > 0 */
    int32_t q_len;              /* T, query tokens per request; 0 reads as 1 (see "Several query tokens") */
} moska_problem_t;

/* Bytes of device workspace that moska_route, moska_bucket, moska_shared_attn and
 * moska_unique_attn may need for this problem (one buffer of this size serves all of them
 * when they run on one stream).  out: host pointer. */
int moska_workspace_bytes(const moska_problem_t *p, size_t *out);

/* Router (Sec. III-B).  score[b,h,c] = (sum over the G query heads of group h of Q[b,hq,:])
 * . E[h,c,:], accumulated in fp64; ids[b,h,0..k-1] are the k best chunks in the order
 * (score descending, chunk id ascending).
 *   Q [B,Hq,D] q_dtype, E [Hkv,C,D] q_dtype (precomputed chunk embeddings),
 *   ids [B,Hkv,k] int32 out, scores [B,Hkv,k] f32 out or NULL (scores of the selected).
 * ws: moska_workspace_bytes (holds all B*Hkv*C scores between scoring and selection).
 * Supports C + D <= 16384. */
int moska_route(const moska_problem_t *p, const void *Q, const void *E,
                int32_t *ids, float *scores, void *ws, size_t ws_bytes, void *stream);

/* Query aggregation (Sec. III-A).  Item (b,h,j) -- slot j of request b on KV head h -- has
 * index b*k+j and falls into bucket h*C + ids[b,h,j].
 *   bucket_off [Hkv*C+1] int32 out: exclusive prefix sum of bucket sizes,
 *   bucket_items [B*Hkv*k] int32 out: the item indices of each bucket, ascending.
 * Deterministic, no atomics.  ids must hold values in [0,C); a chunk named twice for one (request,
 * KV head) gives two items of the same bucket, each served through its own slot.
 * ws: moska_workspace_bytes. */
int moska_bucket(const moska_problem_t *p, const int32_t *ids,
                 int32_t *bucket_off, int32_t *bucket_items,
                 void *ws, size_t ws_bytes, void *stream);

/* Shared KV Attention (Sec. III-A).  For every non-empty bucket (h,c) the query rows of its
 * items (G rows per item) are gathered into one matrix and attend to chunk c of KV head h
 * in one pass over that chunk's K and V; each row's result goes to the slot it was routed
 * through:  part_O[b,hq,j,:], part_LSE[b,hq,j]  for j < k.
 *   Ks, Vs [C,Hkv,L,D] shared_kv_dtype; scale_k, scale_v [C,Hkv] f32 dequantisation
 *   factors (x = scale * stored), required for FP8, NULL otherwise;
 *   bucket_off / bucket_items from moska_bucket; if bucket_off is NULL the grouping is
 *   computed here from ids (then ids must be non-NULL; otherwise ids is not read).
 *   part_O [B,Hq,k+1,D] f32, part_LSE [B,Hq,k+1] f32: slots 0..k-1 are written. */
int moska_shared_attn(const moska_problem_t *p, const void *Q, const void *Ks, const void *Vs,
                      const float *scale_k, const float *scale_v, const int32_t *ids,
                      const int32_t *bucket_off, const int32_t *bucket_items,
                      float *part_O, float *part_LSE, void *ws, size_t ws_bytes, void *stream);

/* Unique KV Attention (Sec. III-A).  Row (b,hq) attends to Ku/Vu[b,hq/G,0:unique_len[b]].
 *   Ku, Vu [B,Hkv,U_max,D] q_dtype; unique_len [B] int32 in [0,U_max], or NULL = U_max.
 *   Writes slot k of part_O / part_LSE. */
int moska_unique_attn(const moska_problem_t *p, const void *Q, const void *Ku, const void *Vu,
                      const int32_t *unique_len, float *part_O, float *part_LSE,
                      void *ws, size_t ws_bytes, void *stream);

/* Combination (Fig. 2(b)).  m = max_p LSE_p, w_p = exp(LSE_p - m),
 * O = sum_p w_p O_p / sum_p w_p, LSE = m + ln sum_p w_p over the P = k+1 slots; slots with
 * LSE = -inf weigh nothing, a row whose slots are all empty gives O = 0, LSE = -inf.
 *   O [B,Hq,D] q_dtype out (bf16: round to nearest even), LSE [B,Hq] f32 out or NULL. */
int moska_merge(const moska_problem_t *p, const float *part_O, const float *part_LSE,
                void *O, float *LSE, void *stream);

/* The five calls above in order on one stream (route -> bucket -> shared -> unique ->
 * merge); every intermediate is a caller-owned buffer with the shape given above. */
int moska_decode_step(const moska_problem_t *p, const void *Q, const void *E,
                      const void *Ks, const void *Vs, const float *scale_k, const float *scale_v,
                      const void *Ku, const void *Vu, const int32_t *unique_len,
                      int32_t *ids, int32_t *bucket_off, int32_t *bucket_items,
                      float *part_O, float *part_LSE, void *O, float *LSE,
                      void *ws, size_t ws_bytes, void *stream);

/* moska_decode_step for callers that cannot allocate a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The workspace is a static array of
 * MOSKA_STATIC_SCRATCH_BYTES in the library's own device memory (each GPU the library runs on
 * holds one until the process ends); the call allocates and frees nothing.  Inputs, outputs and
 * results are those of moska_decode_step (the same kernels run).
 *   - A problem whose moska_workspace_bytes exceeds MOSKA_STATIC_SCRATCH_BYTES is rejected with
 *     MOSKA_ERR_SCRATCH_LIMIT before anything is launched.
 *   - The array's device address is looked up on the first call on each GPU; make that call
 *     outside stream capture.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two host threads) race.  Nothing in it has to be cleared between calls. */
#define MOSKA_STATIC_SCRATCH_BYTES (16u << 20)
int moska_decode_step_static(const moska_problem_t *p, const void *Q, const void *E,
                             const void *Ks, const void *Vs, const float *scale_k, const float *scale_v,
                             const void *Ku, const void *Vu, const int32_t *unique_len,
                             int32_t *ids, int32_t *bucket_off, int32_t *bucket_items,
                             float *part_O, float *part_LSE, void *O, float *LSE, void *stream);

/* Offline construction of the shared store (Sec. III-A: pre-computed shared KV caches;
 * Sec. III-B: precomputed chunk embeddings).  Not part of the decode step.
 *
 * moska_chunk_embeddings: E[h,c,:] = mean over the L stored keys of chunk c on KV head h
 * (times scale_k[c,h] for an FP8 store), accumulated in fp64, rounded to q_dtype.
 *   Ks [C,Hkv,L,D] shared_kv_dtype, scale_k [C,Hkv] f32 (FP8 only, else NULL), E [Hkv,C,D] q_dtype out.
 *
 * moska_quantize_shared: per (chunk, KV head) block scale = max|x| / 448 (at least 1e-30) and
 * X8 = round-to-nearest-even e4m3fn of x / scale, saturating; both divisions in f32.
 *   X [C,Hkv,L,D] bf16 (q_dtype must be BF16, shared_kv_dtype FP8), X8 same shape fp8 out,
 *   scale [C,Hkv] f32 out.  Call once for K and once for V. */
int moska_chunk_embeddings(const moska_problem_t *p, const void *Ks, const float *scale_k, void *E, void *stream);
int moska_quantize_shared(const moska_problem_t *p, const void *X, void *X8, float *scale, void *stream);

/* Static description of a status code. */
const char *moska_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MOSKA_H */
