// moska_merge: log-sum-exp combination of the k shared partials and the unique partial
// (the combination step of Fig. 2(b)).  One wavefront per query row; lane l owns output
// columns l, l+64, ...  The kernel reads P*(D+1) floats and writes D values per row: it is
// bound by HBM traffic on the partials.
#include "moska_internal.h"

namespace moska {
namespace {

template <int OD>
__global__ __launch_bounds__(256) void merge_kernel(const float *__restrict__ part_O,
                                                     const float *__restrict__ part_LSE, void *__restrict__ O,
                                                     float *__restrict__ LSE, int64_t rows, int P, int D) {
    const int lane = threadIdx.x % kWave;
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (r >= rows) return;
    const float *lse = part_LSE + r * P;
    float m = -INFINITY;
    for (int j = 0; j < P; ++j) m = fmaxf(m, lse[j]);
    float wsum = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (m != -INFINITY) {
        for (int j = 0; j < P; ++j) {
            const float lj = lse[j];
            if (lj == -INFINITY) continue;             // an empty slot's O is never read
            const float w = expf(lj - m);
            wsum += w;
            const float *o = part_O + (r * P + j) * D;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (lane + kWave * i < D) acc[i] = fmaf(w, o[lane + kWave * i], acc[i]);
        }
    }
    const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int d = lane + kWave * i;
        if (d < D) {
            const float v = acc[i] * inv;
            if constexpr (OD == MOSKA_BF16) ((uint16_t *)O)[r * D + d] = (uint16_t)f32_to_bf16_bits(v);
            else ((float *)O)[r * D + d] = v;
        }
    }
    if (LSE && lane == 0) LSE[r] = wsum > 0.f ? m + logf(wsum) : -INFINITY;
}

}  // namespace

int launch_merge(const moska_problem_t &p, const float *part_O, const float *part_LSE, void *O, float *LSE,
                 hipStream_t s) {
    const int64_t rows = (int64_t)p.B * p.Hq;
    const unsigned grid = (unsigned)((rows + 3) / 4);
    auto kern = p.q_dtype == MOSKA_BF16 ? merge_kernel<MOSKA_BF16> : merge_kernel<MOSKA_F32>;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, s, part_O, part_LSE, O, LSE, rows, p.k + 1, p.D);
    return hip_status(hipGetLastError());
}

}  // namespace moska
