// moska_route: chunk scoring and top-k selection (paper Sec. III-B).
//
// One 64-lane wavefront owns one (request, KV head) pair.  Lane l scores chunks l, l+64, ...
// against the group-summed query with fp64 FMAs (products of f32 or bf16 inputs are exact in
// fp64, so scores agree with an fp64 reference to rounding order), turns each score into an
// order-preserving 64-bit key kept in LDS, and the wave then extracts the k best with k rounds
// of a butterfly arg-max over (key descending, chunk id ascending).  The work is a few MB and
// a few GFLOP: it is launch/latency bound, far from any roofline.
#include "moska_internal.h"

namespace moska {
namespace {

__device__ __forceinline__ uint64_t order_key(double s) {
    s = s + 0.0;                                   // -0.0 and +0.0 must tie
    uint64_t u = (uint64_t)__double_as_longlong(s);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double key_to_score(uint64_t k) {
    uint64_t u = (k >> 63) ? (k & 0x7FFFFFFFFFFFFFFFull) : ~k;
    return __longlong_as_double((long long)u);
}

// true if (ka,ca) should be selected before (kb,cb)
__device__ __forceinline__ bool before(uint64_t ka, int ca, uint64_t kb, int cb) {
    return ka > kb || (ka == kb && ca < cb);
}

template <int QD>
__global__ __launch_bounds__(256) void route_kernel(const void *__restrict__ Q, const void *__restrict__ E,
                                                     int32_t *__restrict__ ids, float *__restrict__ scores,
                                                     int B, int Hq, int Hkv, int D, int C, int k, int W) {
    extern __shared__ double smem[];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int64_t rows = (int64_t)B * Hkv;
    int64_t r = (int64_t)blockIdx.x * W + wave;    // r = h*B + b: the waves of a block share E[h]
    const bool active = r < rows;
    if (!active) r = rows - 1;                     // compute redundantly, write nothing
    const int h = (int)(r / B), b = (int)(r % B), G = Hq / Hkv;
    double *qs = smem + (size_t)wave * (D + C);
    uint64_t *keys = (uint64_t *)(qs + D);

    for (int d = lane; d < D; d += kWave) {
        double a = 0.0;
        for (int g = 0; g < G; ++g) a += (double)load_f32<QD>(Q, ((int64_t)b * Hq + h * G + g) * D + d);
        qs[d] = a;
    }
    __syncthreads();

    for (int c = lane; c < C; c += kWave) {
        const int64_t base = ((int64_t)h * C + c) * D;
        double a = 0.0;
        if constexpr (QD == MOSKA_BF16) {
            const uint4 *row = (const uint4 *)((const uint16_t *)E + base);
            for (int d8 = 0; d8 < D / 8; ++d8) {
                const uint4 v = row[d8];
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a = fma(qs[d8 * 8 + 2 * i], (double)__uint_as_float(w[i] << 16), a);
                    a = fma(qs[d8 * 8 + 2 * i + 1], (double)__uint_as_float(w[i] & 0xFFFF0000u), a);
                }
            }
        } else {
            const float4 *row = (const float4 *)((const float *)E + base);
            for (int d4 = 0; d4 < D / 4; ++d4) {
                const float4 v = row[d4];
                a = fma(qs[d4 * 4 + 0], (double)v.x, a);
                a = fma(qs[d4 * 4 + 1], (double)v.y, a);
                a = fma(qs[d4 * 4 + 2], (double)v.z, a);
                a = fma(qs[d4 * 4 + 3], (double)v.w, a);
            }
        }
        keys[c] = order_key(a);
    }
    __syncthreads();

    // each lane remembers the best of its own chunks; only the round's winner rescans
    auto rescan = [&](uint64_t &bk, int &bc) {
        bk = 0;                                    // 0 is below every real key
        bc = 0x7FFFFFFF;
        for (int c = lane; c < C; c += kWave) {
            const uint64_t kk = keys[c];
            if (kk > bk) { bk = kk; bc = c; }
        }
    };
    uint64_t bk;
    int bc;
    rescan(bk, bc);
    for (int t = 0; t < k; ++t) {
        uint64_t wk = bk;
        int wc = bc;
#pragma unroll
        for (int m = 1; m < kWave; m <<= 1) {
            const uint64_t ok = __shfl_xor(wk, m);
            const int oc = __shfl_xor(wc, m);
            if (before(ok, oc, wk, wc)) { wk = ok; wc = oc; }
        }
        if (lane == (wc & (kWave - 1))) {
            keys[wc] = 0;
            rescan(bk, bc);
        }
        if (active && lane == 0) {
            const int64_t o = ((int64_t)b * Hkv + h) * k + t;
            ids[o] = wc;
            if (scores) scores[o] = (float)key_to_score(wk);
        }
    }
}

}  // namespace

int launch_route(const moska_problem_t &p, const void *Q, const void *E, int32_t *ids, float *scores,
                 hipStream_t s) {
    const size_t per_wave = (size_t)(p.D + p.C) * sizeof(double);
    int W = (int)((140u * 1024u) / per_wave);
    if (W < 1) return MOSKA_ERR_UNSUPPORTED;
    if (W > 4) W = 4;
    const size_t lds = per_wave * W;
    const int64_t rows = (int64_t)p.B * p.Hkv;
    const unsigned grid = (unsigned)((rows + W - 1) / W);
    auto kern = p.q_dtype == MOSKA_BF16 ? route_kernel<MOSKA_BF16> : route_kernel<MOSKA_F32>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return MOSKA_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(W * kWave), lds, s, Q, E, ids, scores, p.B, p.Hq, p.Hkv, p.D, p.C,
                       p.k, W);
    return hip_status(hipGetLastError());
}

}  // namespace moska
