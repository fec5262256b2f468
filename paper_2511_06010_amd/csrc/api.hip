// C entry points: host-side validation, workspace carving and kernel dispatch.
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "moska_internal.h"

namespace moska {

// Development builds (-DMOSKA_TUNING) take overrides of the launch heuristics from the environment, each
// read once per process; the library as shipped reads no environment and holds no state.
#ifdef MOSKA_TUNING
int tuning_env(const char *name, int dflt) {
    const char *e = std::getenv(name);
    return e && *e ? std::atoi(e) : dflt;
}
#endif

bool use_mfma_path(const moska_problem_t &p) {
    static const bool force_generic = tuning_env("MOSKA_FORCE_GENERIC", 0) == 1;
    return !force_generic && p.q_dtype == MOSKA_BF16 && p.D == 128;
}

SharedPlan shared_plan(const moska_problem_t &p) {
    if (!use_mfma_path(p)) return SharedPlan{0, 0};          // the vector-ALU kernel serves 16-row tiles
    // smallest / largest tile class (0..4 = 16, 32, 64, 128, 256 rows)
    static const int cmin_env = tuning_env("MOSKA_SHARED_CMIN", 0), cmax_env = tuning_env("MOSKA_SHARED_CMAX", kNumClasses - 1);
    SharedPlan pl{cmin_env, cmax_env};
    if (pl.cmin < 0) pl.cmin = 0;
    if (pl.cmax > kNumClasses - 1) pl.cmax = kNumClasses - 1;
    if (pl.cmin > pl.cmax) pl.cmin = pl.cmax;
    return pl;
}

// a positive override replaces the heuristic
static int env_splits(const char *name, int limit) {
    const int v = tuning_env(name, 0);
    return v < 1 ? 0 : v > limit ? limit : v;
}

int unique_splits(const moska_problem_t &p) {
    if (!use_mfma_path(p)) return 1;
    static const int forced = env_splits("MOSKA_UNIQUE_SPLITS", 32);
    if (forced) return p.U_max >= 64 * forced ? forced : 1;
    const int R = q_len(p) * (p.Hq / p.Hkv);                   // query rows per (request, KV head)
    const int rows_per_wg = R <= 16 ? 16 : R <= 32 ? 32 : 64;
    const int64_t wgs = (int64_t)p.B * p.Hkv * ((R + rows_per_wg - 1) / rows_per_wg);
    if (wgs >= 512 || p.U_max < 512) return 1;
    int64_t n = (1024 + wgs - 1) / wgs;                     // aim at ~1024 workgroups ...
    if (n > p.U_max / 256) n = p.U_max / 256;               // ... of at least 256 keys each
    if (n > 32) n = 32;
    return n < 1 ? 1 : (int)n;
}

int shared_splits(const moska_problem_t &p) {
    if (!use_mfma_path(p)) return 1;
    static const int forced = env_splits("MOSKA_SHARED_SPLITS", 16);
    if (forced) return p.L >= 64 * forced ? forced : 1;
    const int64_t items = (int64_t)p.B * q_len(p) * p.Hkv * p.k, nb = (int64_t)p.Hkv * p.C;
    const int64_t nbe = items < nb ? items : nb;            // buckets that can be non-empty
    if (nbe > 256 || p.L < 1024) return 1;                  // one workgroup per compute unit already
    // tiles hold at most 256 rows, so many rows in few buckets also mean many workgroups
    const int64_t by_rows = items * (p.Hq / p.Hkv) / 256;
    const int64_t wgs = nbe > by_rows ? nbe : by_rows;      // workgroups the launch has at least
    int64_t n = (512 + wgs - 1) / wgs;                      // aim at ~512 workgroups ...
    if (n > p.L / 512) n = p.L / 512;                       // ... of at least 512 keys each
    if (n > 16) n = 16;
    return n < 1 ? 1 : (int)n;
}

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

Workspace carve_workspace(const moska_problem_t &p, void *ws) {
    Workspace w;
    const size_t Bq = (size_t)p.B * q_len(p);               // query tokens
    const size_t items = Bq * p.Hkv * p.k, nb = (size_t)p.Hkv * p.C;
    // bound valid for every plan: at most one remainder tile per class and bucket plus the full tiles
    const size_t tmax = (size_t)(4 * (items < nb ? items : nb) + (items * (size_t)(p.Hq / p.Hkv)) / 16 + 8);
    char *base = (char *)ws;
    size_t o = 0;
    w.tile_hdr = (int32_t *)(base + o); o += align_up(8 * sizeof(int32_t));
    w.tiles = (int32_t *)(base + o);    o += align_up(2 * tmax * sizeof(int32_t));
    w.rank = (int32_t *)(base + o);     o += align_up(items * sizeof(int32_t));
    const int nsl = bucket_slices(per_token(p));
    w.slice_hist = (int32_t *)(base + o); o += align_up(nsl > 1 ? nb * nsl * sizeof(int32_t) : 0);
    w.off = (int32_t *)(base + o);      o += align_up((nb + 1) * sizeof(int32_t));
    w.items = (int32_t *)(base + o);    o += align_up(items * sizeof(int32_t));
    const int ns = unique_splits(p);
    const size_t srows = ns > 1 ? Bq * p.Hq * ns : 0;
    w.split_O = (float *)(base + o);    o += align_up(srows * p.D * sizeof(float));
    w.split_LSE = (float *)(base + o);  o += align_up(srows * sizeof(float));
    const int nss = shared_splits(p);
    const size_t ssrows = nss > 1 ? Bq * p.Hq * p.k * nss : 0;
    w.ssplit_O = (float *)(base + o);   o += align_up(ssrows * p.D * sizeof(float));
    w.ssplit_LSE = (float *)(base + o); o += align_up(ssrows * sizeof(float));
    w.route_keys = (uint64_t *)(base + o); o += align_up(Bq * p.Hkv * p.C * sizeof(uint64_t));
    w.bytes = o;
    return w;
}

static int check_problem(const moska_problem_t *p) {
    if (!p) return MOSKA_ERR_INVALID_ARG;
    if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->D < 1 || p->C < 1 || p->L < 1 || p->k < 1 || p->U_max < 0 ||
        p->q_len < 0)
        return MOSKA_ERR_INVALID_ARG;
    if (p->Hq % p->Hkv != 0 || p->k > p->C || !(p->scale > 0.f)) return MOSKA_ERR_INVALID_ARG;
    if (p->D % 16 != 0 || p->D > 256) return MOSKA_ERR_UNSUPPORTED;
    const bool f32 = p->q_dtype == MOSKA_F32 && p->shared_kv_dtype == MOSKA_F32;
    const bool b16 = p->q_dtype == MOSKA_BF16 &&
                     (p->shared_kv_dtype == MOSKA_BF16 || p->shared_kv_dtype == MOSKA_FP8_E4M3);
    if (!f32 && !b16) return MOSKA_ERR_UNSUPPORTED;
    if ((int64_t)p->C + p->D > 16384) return MOSKA_ERR_UNSUPPORTED;
    // byte offsets inside one chunk / one request's unique store are 32-bit in the kernels
    if ((int64_t)p->L * p->D * 4 >= (int64_t)1 << 32 || (int64_t)p->U_max * p->D * 4 >= (int64_t)1 << 32)
        return MOSKA_ERR_UNSUPPORTED;
    // index arithmetic inside one head uses int32 item numbers
    const int64_t Bq = (int64_t)p->B * q_len(*p);
    if (Bq * p->Hkv * p->k > (int64_t)1 << 30 || Bq * p->Hq * (p->k + 1) > (int64_t)1 << 30) return MOSKA_ERR_UNSUPPORTED;
    return MOSKA_OK;
}

// Workspace of moska_decode_step_static: one array per GPU, in the library's own device memory for
// as long as the process lives.  `scratch` is a host-side stand-in for the symbol, not a device
// address; its address on the current device is looked up once per device and kept in scratch_ptr.
constexpr size_t kScratchBytes = (size_t)MOSKA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static void *scratch_ptr[kMaxDevices];
static std::mutex scratch_mutex;

static int scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOSKA_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MOSKA_ERR_HIP;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return MOSKA_OK;
}

}  // namespace moska

using namespace moska;

extern "C" {

const char *moska_status_string(int status) {
    switch (status) {
    case MOSKA_OK: return "ok";
    case MOSKA_ERR_INVALID_ARG: return "invalid argument";
    case MOSKA_ERR_UNSUPPORTED: return "unsupported dtype or size";
    case MOSKA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MOSKA_ERR_HIP: return "HIP runtime error";
    case MOSKA_ERR_SCRATCH_LIMIT: return "problem needs more workspace than the static scratch buffer holds";
    default: return "unknown status";
    }
}

int moska_workspace_bytes(const moska_problem_t *p, size_t *out) {
    if (!out) return MOSKA_ERR_INVALID_ARG;
    if (int rc = check_problem(p)) return rc;
    *out = carve_workspace(*p, nullptr).bytes;
    return MOSKA_OK;
}

int moska_route(const moska_problem_t *p, const void *Q, const void *E, int32_t *ids, float *scores, void *ws,
                size_t ws_bytes, void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!Q || !E || !ids || !ws) return MOSKA_ERR_INVALID_ARG;
    const Workspace w = carve_workspace(*p, ws);
    if (ws_bytes < w.bytes) return MOSKA_ERR_WORKSPACE_TOO_SMALL;
    return launch_route(per_token(*p), Q, E, ids, scores, w.route_keys, (hipStream_t)stream);
}

int moska_bucket(const moska_problem_t *p, const int32_t *ids, int32_t *bucket_off, int32_t *bucket_items, void *ws,
                 size_t ws_bytes, void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!ids || !bucket_off || !bucket_items || !ws) return MOSKA_ERR_INVALID_ARG;
    const Workspace w = carve_workspace(*p, ws);
    if (ws_bytes < w.bytes) return MOSKA_ERR_WORKSPACE_TOO_SMALL;
    return launch_bucket(per_token(*p), ids, bucket_off, bucket_items, w.rank, w.slice_hist, (hipStream_t)stream);
}

int moska_shared_attn(const moska_problem_t *p, const void *Q, const void *Ks, const void *Vs, const float *scale_k,
                      const float *scale_v, const int32_t *ids, const int32_t *bucket_off,
                      const int32_t *bucket_items, float *part_O, float *part_LSE, void *ws, size_t ws_bytes,
                      void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!Q || !Ks || !Vs || !part_O || !part_LSE || !ws) return MOSKA_ERR_INVALID_ARG;
    const bool fp8 = p->shared_kv_dtype == MOSKA_FP8_E4M3;
    if (fp8 && (!scale_k || !scale_v)) return MOSKA_ERR_INVALID_ARG;
    if (!fp8) scale_k = scale_v = nullptr;
    if (bucket_off ? !bucket_items : !ids) return MOSKA_ERR_INVALID_ARG;
    const Workspace w = carve_workspace(*p, ws);
    if (ws_bytes < w.bytes) return MOSKA_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)stream;
    if (!bucket_off) {
        if (int rc = launch_bucket(per_token(*p), ids, w.off, w.items, w.rank, w.slice_hist, s)) return rc;
        bucket_off = w.off;
        bucket_items = w.items;
    }
    const SharedPlan pl = shared_plan(*p);
    const moska_problem_t f = per_token(*p);
    if (int rc = launch_tile_list(f, bucket_off, pl, w.tile_hdr, w.tiles, s)) return rc;
    const int nss = shared_splits(*p);
    SharedArgs a{Q, Ks, Vs, scale_k, scale_v, bucket_off, bucket_items, w.tile_hdr, w.tiles, part_O, part_LSE,
                 nss > 1 ? w.ssplit_O : nullptr, nss > 1 ? w.ssplit_LSE : nullptr, nss};
    return use_mfma_path(f) ? launch_shared_mfma(f, a, pl, s) : launch_shared_generic(f, a, pl, s);
}

int moska_unique_attn(const moska_problem_t *p, const void *Q, const void *Ku, const void *Vu,
                      const int32_t *unique_len, float *part_O, float *part_LSE, void *ws, size_t ws_bytes,
                      void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!Q || !part_O || !part_LSE) return MOSKA_ERR_INVALID_ARG;
    if (p->U_max > 0 && (!Ku || !Vu)) return MOSKA_ERR_INVALID_ARG;
    const int ns = unique_splits(*p);
    UniqueArgs a{Q, Ku, Vu, unique_len, part_O, part_LSE, nullptr, nullptr, ns};
    if (ns > 1) {
        if (!ws) return MOSKA_ERR_INVALID_ARG;
        const Workspace w = carve_workspace(*p, ws);
        if (ws_bytes < w.bytes) return MOSKA_ERR_WORKSPACE_TOO_SMALL;
        a.split_O = w.split_O;
        a.split_LSE = w.split_LSE;
    }
    hipStream_t s = (hipStream_t)stream;
    return use_mfma_path(*p) ? launch_unique_mfma(*p, a, s) : launch_unique_generic(*p, a, s);
}

int moska_merge(const moska_problem_t *p, const float *part_O, const float *part_LSE, void *O, float *LSE,
                void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!part_O || !part_LSE || !O) return MOSKA_ERR_INVALID_ARG;
    return launch_merge(per_token(*p), part_O, part_LSE, O, LSE, (hipStream_t)stream);
}

int moska_decode_step(const moska_problem_t *p, const void *Q, const void *E, const void *Ks, const void *Vs,
                      const float *scale_k, const float *scale_v, const void *Ku, const void *Vu,
                      const int32_t *unique_len, int32_t *ids, int32_t *bucket_off, int32_t *bucket_items,
                      float *part_O, float *part_LSE, void *O, float *LSE, void *ws, size_t ws_bytes, void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!Q || !E || !Ks || !Vs || !ids || !bucket_off || !bucket_items || !part_O || !part_LSE || !O || !ws)
        return MOSKA_ERR_INVALID_ARG;
    if (p->U_max > 0 && (!Ku || !Vu)) return MOSKA_ERR_INVALID_ARG;
    if (p->shared_kv_dtype == MOSKA_FP8_E4M3 && (!scale_k || !scale_v)) return MOSKA_ERR_INVALID_ARG;
    if (ws_bytes < carve_workspace(*p, ws).bytes) return MOSKA_ERR_WORKSPACE_TOO_SMALL;
    if (int rc = moska_route(p, Q, E, ids, nullptr, ws, ws_bytes, stream)) return rc;
    if (int rc = moska_bucket(p, ids, bucket_off, bucket_items, ws, ws_bytes, stream)) return rc;
    if (int rc = moska_shared_attn(p, Q, Ks, Vs, scale_k, scale_v, ids, bucket_off, bucket_items, part_O, part_LSE, ws,
                                   ws_bytes, stream))
        return rc;
    if (int rc = moska_unique_attn(p, Q, Ku, Vu, unique_len, part_O, part_LSE, ws, ws_bytes, stream)) return rc;
    return moska_merge(p, part_O, part_LSE, O, LSE, stream);
}

int moska_decode_step_static(const moska_problem_t *p, const void *Q, const void *E, const void *Ks, const void *Vs,
                             const float *scale_k, const float *scale_v, const void *Ku, const void *Vu,
                             const int32_t *unique_len, int32_t *ids, int32_t *bucket_off, int32_t *bucket_items,
                             float *part_O, float *part_LSE, void *O, float *LSE, void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (carve_workspace(*p, nullptr).bytes > kScratchBytes) return MOSKA_ERR_SCRATCH_LIMIT;
    void *ws = nullptr;
    if (int rc = scratch_of_current_device(&ws)) return rc;
    // nothing in the workspace has to start at zero: every region is written before it is read
    return moska_decode_step(p, Q, E, Ks, Vs, scale_k, scale_v, Ku, Vu, unique_len, ids, bucket_off, bucket_items,
                             part_O, part_LSE, O, LSE, ws, kScratchBytes, stream);
}

int moska_chunk_embeddings(const moska_problem_t *p, const void *Ks, const float *scale_k, void *E, void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!Ks || !E) return MOSKA_ERR_INVALID_ARG;
    const bool fp8 = p->shared_kv_dtype == MOSKA_FP8_E4M3;
    if (fp8 && !scale_k) return MOSKA_ERR_INVALID_ARG;
    return launch_chunk_embeddings(*p, Ks, fp8 ? scale_k : nullptr, E, (hipStream_t)stream);
}

int moska_quantize_shared(const moska_problem_t *p, const void *X, void *X8, float *scale, void *stream) {
    if (int rc = check_problem(p)) return rc;
    if (!X || !X8 || !scale) return MOSKA_ERR_INVALID_ARG;
    if (p->q_dtype != MOSKA_BF16 || p->shared_kv_dtype != MOSKA_FP8_E4M3) return MOSKA_ERR_UNSUPPORTED;
    return launch_quantize_fp8(*p, X, X8, scale, (hipStream_t)stream);
}

}  // extern "C"
