// Shared and unique attention on the fp32 vector ALUs, any supported dtype and head size.
//
// This is the path of the fp32 configuration (results within 1e-5 relative of an fp64
// reference need fp32 products and an accurate exp, so no bf16 MFMA) and the fallback for
// head sizes the MFMA kernels do not cover.  It still follows the method: a workgroup takes up
// to 16 query rows that attend to the SAME key set -- the rows of one bucket for Shared KV
// Attention (Sec. III-A), the G heads of one request for Unique KV Attention -- stages each
// 64-key tile of K and V in LDS once, and all rows consume it.
//
// Thread (r, x) of the 256 (r = row 0..15, x = 0..15): scores keys x, x+16, x+32, x+48 of the
// tile for row r, then accumulates output columns x, x+16, ... for row r.
#include "moska_internal.h"

namespace moska {
namespace {

constexpr int TR = 16;      // rows per workgroup
constexpr int TK = 64;      // keys per tile
constexpr int MAXD16 = 16;  // D <= 256

struct RowSet {             // the rows a workgroup serves and the keys they attend to
    int nrows;
    int64_t kv_base;        // element offset of key 0 in K and V
    int nkeys;              // keys of the set; row r sees the first lim[r] <= nkeys of them (lim = nullptr: all)
    const int *lim;         // LDS array
    float kmul, vmul;
};

template <int QD, int KD>
__device__ void attend_tile_rows(const RowSet &rs, const int64_t *q_off, const int64_t *o_row, const void *Q,
                                 const void *K, const void *V, float scale, int D, float *part_O, float *part_LSE,
                                 int P) {
    // q_off[r]: element offset of row r's query; o_row[r]: (b*Hq+hq)*P + slot (LDS arrays)
    extern __shared__ float smem[];
    const int DP = D + 1;
    float *Qs = smem;                    // [TR][DP]
    float *Ks = Qs + TR * DP;            // [TK][DP]
    float *Vs = Ks + TK * DP;            // [TK][DP]
    float *Ps = Vs + TK * DP;            // [TR][TK+1]
    const int tid = threadIdx.x, r = tid / 16, x = tid % 16;
    const int nd = D / 16;

    for (int i = tid; i < TR * D; i += 256) {
        const int rr = i / D, d = i - rr * D;
        Qs[rr * DP + d] = rr < rs.nrows ? load_f32<QD>(Q, q_off[rr] + d) : 0.f;
    }
    float acc[MAXD16];
#pragma unroll
    for (int i = 0; i < MAXD16; ++i) acc[i] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float sc = scale * rs.kmul;
    const int mylim = rs.lim ? rs.lim[r] : rs.nkeys;

    for (int k0 = 0; k0 < rs.nkeys; k0 += TK) {
        __syncthreads();                 // previous tile fully consumed (and Qs written)
        const int nk = min(TK, rs.nkeys - k0);
        for (int i = tid; i < TK * D; i += 256) {
            const int kk = i / D, d = i - kk * D;
            const bool ok = kk < nk;
            const int64_t g = rs.kv_base + (int64_t)(k0 + kk) * D + d;
            Ks[kk * DP + d] = ok ? load_f32<KD>(K, g) : 0.f;
            Vs[kk * DP + d] = ok ? load_f32<KD>(V, g) : 0.f;
        }
        __syncthreads();
        float s[4], tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int kk = x + 16 * i;
            float a = 0.f;
            for (int d = 0; d < D; ++d) a = fmaf(Qs[r * DP + d], Ks[kk * DP + d], a);
            s[i] = k0 + kk < mylim ? a * sc : -INFINITY;
            tmax = fmaxf(tmax, s[i]);
        }
#pragma unroll
        for (int w = 1; w < 16; w <<= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, w, 16));
        const float mn = fmaxf(m, tmax);             // -inf only while the row has seen no key
        const float alpha = m == -INFINITY ? 0.f : expf(m - mn);
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float pv = s[i] == -INFINITY ? 0.f : expf(s[i] - mn);   // masked keys weigh nothing
            Ps[r * (TK + 1) + x + 16 * i] = pv;
            lsum += pv;
        }
#pragma unroll
        for (int w = 1; w < 16; w <<= 1) lsum += __shfl_xor(lsum, w, 16);
        l = l * alpha + lsum;
        m = mn;
#pragma unroll
        for (int i = 0; i < MAXD16; ++i) acc[i] *= alpha;
        __syncthreads();
        for (int kk = 0; kk < nk; ++kk) {
            const float pv = Ps[r * (TK + 1) + kk];
#pragma unroll
            for (int i = 0; i < MAXD16; ++i)
                if (i < nd) acc[i] = fmaf(pv, Vs[kk * DP + x + 16 * i], acc[i]);
        }
    }
    if (r < rs.nrows) {
        const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
        for (int i = 0; i < MAXD16; ++i)
            if (i < nd) part_O[o_row[r] * D + x + 16 * i] = acc[i] * inv * rs.vmul;
        if (x == 0) part_LSE[o_row[r]] = l > 0.f ? m + logf(l) : -INFINITY;
    }
    (void)P;
}

template <int QD, int KD>
__global__ __launch_bounds__(256) void shared_generic_kernel(SharedArgs a, int B, int Hq, int Hkv, int D, int C,
                                                              int L, int k, float scale) {
    __shared__ int64_t q_off[TR], o_row[TR];
    constexpr int MT = TR;
    const int ntiles = a.tile_hdr[1] - a.tile_hdr[0];    // only the 16-row class is in use
    if ((int)blockIdx.x >= ntiles) return;
    const int bkt = a.tiles[2 * blockIdx.x], row0 = a.tiles[2 * blockIdx.x + 1];
    const int h = bkt / C, c = bkt - h * C, G = Hq / Hkv, P = k + 1;
    const int beg = a.off[bkt], rows = (a.off[bkt + 1] - beg) * G;
    RowSet rs;
    rs.nrows = min(MT, rows - row0);
    rs.kv_base = ((int64_t)c * Hkv + h) * L * D;
    rs.nkeys = L;
    rs.lim = nullptr;
    rs.kmul = a.scale_k ? a.scale_k[c * Hkv + h] : 1.f;
    rs.vmul = a.scale_v ? a.scale_v[c * Hkv + h] : 1.f;
    if (threadIdx.x < TR && (int)threadIdx.x < rs.nrows) {
        const int rr = row0 + threadIdx.x;
        const int item = a.items[beg + rr / G], g = rr % G;
        const int b = item / k, j = item - b * k, hq = h * G + g;
        q_off[threadIdx.x] = ((int64_t)b * Hq + hq) * D;
        o_row[threadIdx.x] = ((int64_t)b * Hq + hq) * P + j;
    }
    __syncthreads();
    attend_tile_rows<QD, KD>(rs, q_off, o_row, a.Q, a.Ks, a.Vs, scale, D, a.part_O, a.part_LSE, P);
}

// Rows of a (request, KV head) pair: row t*G + g is query token t, head g of the group; token t
// sees the first len - (T-1-t) keys of the request's context.
template <int QD>
__global__ __launch_bounds__(256) void unique_generic_kernel(UniqueArgs a, int B, int Hq, int Hkv, int D, int U,
                                                              int k, float scale, int T) {
    __shared__ int64_t q_off[TR], o_row[TR];
    __shared__ int lim[TR];
    const int G = Hq / Hkv, P = k + 1, R = T * G, gt = (R + TR - 1) / TR;
    const int bh = blockIdx.x / gt, r0 = (blockIdx.x % gt) * TR;
    const int b = bh / Hkv, h = bh - b * Hkv;
    RowSet rs;
    rs.nrows = min(TR, R - r0);
    rs.kv_base = ((int64_t)b * Hkv + h) * U * D;
    rs.nkeys = a.unique_len ? min(max(a.unique_len[b], 0), U) : U;
    rs.lim = lim;
    rs.kmul = rs.vmul = 1.f;
    if ((int)threadIdx.x < TR) {
        const int r = min(r0 + (int)threadIdx.x, R - 1);
        const int t = r / G, hq = h * G + (r - t * G);
        const int64_t row = ((int64_t)b * T + t) * Hq + hq;
        q_off[threadIdx.x] = row * D;
        o_row[threadIdx.x] = row * P + k;
        lim[threadIdx.x] = max(rs.nkeys - (T - 1 - t), 0);
    }
    __syncthreads();
    attend_tile_rows<QD, QD>(rs, q_off, o_row, a.Q, a.Ku, a.Vu, scale, D, a.part_O, a.part_LSE, P);
}

size_t generic_lds_bytes(int D) { return ((size_t)(TR + 2 * TK) * (D + 1) + (size_t)TR * (TK + 1)) * sizeof(float); }

template <typename Kern>
int set_lds(Kern kern, size_t lds) {
    if (lds <= 48 * 1024) return MOSKA_OK;
    return hip_status(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
}

}  // namespace

int launch_shared_generic(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    if (pl.cmin != 0 || pl.cmax != 0 || class_rows(0) != TR) return MOSKA_ERR_UNSUPPORTED;
    const size_t lds = generic_lds_bytes(p.D);
    const unsigned grid = (unsigned)tiles_bound(p, pl, 0, 0);
    if (grid == 0) return MOSKA_OK;
    void (*kern)(SharedArgs, int, int, int, int, int, int, int, float) = nullptr;
    if (p.q_dtype == MOSKA_F32 && p.shared_kv_dtype == MOSKA_F32) kern = shared_generic_kernel<MOSKA_F32, MOSKA_F32>;
    else if (p.q_dtype == MOSKA_BF16 && p.shared_kv_dtype == MOSKA_BF16) kern = shared_generic_kernel<MOSKA_BF16, MOSKA_BF16>;
    else if (p.q_dtype == MOSKA_BF16 && p.shared_kv_dtype == MOSKA_FP8_E4M3) kern = shared_generic_kernel<MOSKA_BF16, MOSKA_FP8_E4M3>;
    else return MOSKA_ERR_UNSUPPORTED;
    if (int rc = set_lds(kern, lds)) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, a, p.B, p.Hq, p.Hkv, p.D, p.C, p.L, p.k, p.scale);
    return hip_status(hipGetLastError());
}

int launch_unique_generic(const moska_problem_t &p, const UniqueArgs &a, hipStream_t s) {
    const size_t lds = generic_lds_bytes(p.D);
    const int T = q_len(p), R = T * (p.Hq / p.Hkv);
    const unsigned grid = (unsigned)((int64_t)p.B * p.Hkv * ((R + TR - 1) / TR));
    auto kern = p.q_dtype == MOSKA_BF16 ? unique_generic_kernel<MOSKA_BF16> : unique_generic_kernel<MOSKA_F32>;
    if (int rc = set_lds(kern, lds)) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, a, p.B, p.Hq, p.Hkv, p.D, p.U_max, p.k, p.scale, T);
    return hip_status(hipGetLastError());
}

}  // namespace moska
