// Internal declarations shared by the library's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moska.h"

namespace moska {

constexpr int kWave = 64;

// Override of a launch heuristic, for development builds only (-DMOSKA_TUNING: an integer from the named
// environment variable); the library as shipped always gets the default.
#ifdef MOSKA_TUNING
int tuning_env(const char *name, int dflt);
#else
inline int tuning_env(const char *, int dflt) { return dflt; }
#endif

bool use_mfma_path(const moska_problem_t &p);

// Work tiles of Shared KV Attention.  A bucket's rows are cut into tiles of one of five sizes.
// A bucket of M rows becomes full tiles of the largest class in the plan plus one remainder tile of
// the smallest class that holds it, so every bucket's chunk is streamed as few times as possible.
constexpr int kNumClasses = 5;
__host__ __device__ constexpr int class_rows(int c) { return 16 << c; }   // 16, 32, 64, 128, 256
struct SharedPlan {
    int cmin, cmax;          // classes in use
};
SharedPlan shared_plan(const moska_problem_t &p);

// Upper bound on the number of tiles of classes c_lo..c_hi (host-known, sizes the launch grid).  Pure
// counting: a bucket has one remainder tile, there are at most min(items, buckets) non-empty buckets,
// a remainder tile of class c > cmin holds more than class_rows(c-1) rows, and full tiles are of the
// largest class.  It holds for any ids in [0,C), also repeated ones.
inline int64_t tiles_bound(const moska_problem_t &p, const SharedPlan &pl, int c_lo, int c_hi) {
    if (c_lo < pl.cmin) c_lo = pl.cmin;
    if (c_hi > pl.cmax) c_hi = pl.cmax;
    if (c_lo > c_hi) return 0;
    const int64_t items = (int64_t)p.B * p.Hkv * p.k, nb = (int64_t)p.Hkv * p.C;
    const int64_t rows = items * (p.Hq / p.Hkv);
    int64_t rem = items < nb ? items : nb;
    if (c_lo > pl.cmin && rows / (class_rows(c_lo - 1) + 1) < rem) rem = rows / (class_rows(c_lo - 1) + 1);
    return c_hi == pl.cmax ? rem + rows / class_rows(pl.cmax) : rem;
}

// Unique KV Attention splits each request's context over this many workgroups when there are too
// few (request, KV head) pairs to fill the chip (small batches); 1 = no split.
int unique_splits(const moska_problem_t &p);
// Likewise Shared KV Attention splits every chunk's keys over this many workgroups when there are
// too few buckets (few chunks and KV heads); 1 = no split.
int shared_splits(const moska_problem_t &p);

// Workspace layout (int32 units), one region per user:
//   [tile header 8: start of each class in the tile list, total][tile list 2*Tmax]
//   [bucket rank scratch n_items][internal bucket_off NB+1][internal bucket_items n_items]
struct Workspace {
    int32_t *tile_hdr;
    int32_t *tiles;         // (bucket, first row) pairs, grouped by class
    int32_t *rank;          // moska_bucket scratch
    int32_t *slice_hist;    // moska_bucket scratch of the multi-workgroup form: [Hkv][slices][C]
    int32_t *off;           // bucket_off when the caller passes none
    int32_t *items;
    float *split_O;         // [B,Hq,splits,D] partial outputs of a split unique attention
    float *split_LSE;       // [B,Hq,splits]
    float *ssplit_O;        // [B,Hq,k,splits,D] partial outputs of a split shared attention
    float *ssplit_LSE;      // [B,Hq,k,splits]
    uint64_t *route_keys;   // [B,Hkv,C] routing scores as order-preserving keys
    size_t bytes;
};
Workspace carve_workspace(const moska_problem_t &p, void *ws);

int launch_route(const moska_problem_t &p, const void *Q, const void *E, int32_t *ids, float *scores, uint64_t *keys,
                 hipStream_t s);
// Heads with very many items are bucketed by this many workgroups each (1: one workgroup per head);
// p with one query token per request.
int bucket_slices(const moska_problem_t &p);
int launch_bucket(const moska_problem_t &p, const int32_t *ids, int32_t *off, int32_t *items,
                  int32_t *rank_scratch, int32_t *slice_hist, hipStream_t s);
int launch_tile_list(const moska_problem_t &p, const int32_t *off, const SharedPlan &pl, int32_t *hdr,
                     int32_t *tiles, hipStream_t s);

struct SharedArgs {
    const void *Q, *Ks, *Vs;
    const float *scale_k, *scale_v;
    const int32_t *off, *items, *tile_hdr, *tiles;
    float *part_O, *part_LSE;
    float *split_O, *split_LSE;   // workspace of a split run (nsplit > 1)
    int nsplit;
};
struct UniqueArgs {
    const void *Q, *Ku, *Vu;
    const int32_t *unique_len;
    float *part_O, *part_LSE;
    float *split_O, *split_LSE;   // workspace of a split run (nsplit > 1)
    int nsplit;
};
int launch_shared_generic(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s);
int launch_unique_generic(const moska_problem_t &p, const UniqueArgs &a, hipStream_t s);
int launch_shared_mfma(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s);
int launch_unique_mfma(const moska_problem_t &p, const UniqueArgs &a, hipStream_t s);
int launch_merge(const moska_problem_t &p, const float *part_O, const float *part_LSE, void *O, float *LSE,
                 hipStream_t s);

int launch_chunk_embeddings(const moska_problem_t &p, const void *Ks, const float *scale_k, void *E, hipStream_t s);
int launch_quantize_fp8(const moska_problem_t &p, const void *X, void *X8, float *scale, hipStream_t s);

// query tokens per request (0 in the descriptor reads as 1) and in the whole step
inline int q_len(const moska_problem_t &p) { return p.q_len > 0 ? p.q_len : 1; }
// The same step with every query token as a request of its own: what routing, bucketing, shared
// attention and the merge work on (only unique attention needs to know which tokens share a context).
inline moska_problem_t per_token(const moska_problem_t &p) {
    moska_problem_t f = p;
    f.B = p.B * q_len(p);
    f.q_len = 1;
    return f;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? MOSKA_OK : MOSKA_ERR_HIP; }

// ---- storage dtype helpers (device) ----------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// round-to-nearest-even f32 -> bf16 bits (inputs here are finite)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// OCP e4m3fn byte -> f32, exact
__device__ __forceinline__ float fp8_e4m3fn_to_f32(uint32_t b) {
    const uint32_t s = (b & 0x80u) << 24, e = (b >> 3) & 15u, m = b & 7u;
    if (e == 0) return __uint_as_float(s | __float_as_uint((float)m * 0.001953125f));
    return __uint_as_float(s | ((e + 120u) << 23) | (m << 20));   // 0x7F decodes as 480, not NaN: unsupported input
}

template <int DT>
__device__ __forceinline__ float load_f32(const void *p, int64_t i) {
    if constexpr (DT == MOSKA_F32) return ((const float *)p)[i];
    else if constexpr (DT == MOSKA_BF16) return bf16_bits_to_f32(((const uint16_t *)p)[i]);
    else return fp8_e4m3fn_to_f32(((const uint8_t *)p)[i]);
}

}  // namespace moska
