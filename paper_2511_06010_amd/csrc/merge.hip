// moska_merge: log-sum-exp combination of the k shared partials and the unique partial
// (the combination step of Fig. 2(b)).  D/4 threads per query row, each owning four adjacent
// output columns (16-byte loads of every partial).  The kernel reads P*(D+1) floats and writes D
// values per row: it is bound by HBM traffic on the partials.
#include "moska_internal.h"

namespace moska {
namespace {

template <int OD>
__global__ __launch_bounds__(256) void merge_kernel(const float *__restrict__ part_O,
                                                     const float *__restrict__ part_LSE, void *__restrict__ O,
                                                     float *__restrict__ LSE, int64_t rows, int P, int D) {
    const int tpr = D / 4;                                  // threads per row (D is a multiple of 16)
    const int rpb = 256 / tpr;                              // rows per block
    const int t = threadIdx.x % tpr;
    const int64_t r = (int64_t)blockIdx.x * rpb + threadIdx.x / tpr;
    if (threadIdx.x >= rpb * tpr || r >= rows) return;
    const float *lse = part_LSE + r * P;
    float m = -INFINITY;
    for (int j = 0; j < P; ++j) m = fmaxf(m, lse[j]);
    float wsum = 0.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    if (m != -INFINITY) {
        // four slots per round, their loads issued together; an empty slot's O may hold anything:
        // it is loaded (the address is valid) but never enters the arithmetic
        const float *po = part_O + r * P * D + 4 * t;
        for (int j0 = 0; j0 < P; j0 += 4) {
            float4 o[4];
            float w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = min(j0 + u, P - 1);
                o[u] = *(const float4 *)(po + (int64_t)j * D);
                const float lj = lse[j];
                w[u] = (j0 + u < P && lj != -INFINITY) ? expf(lj - m) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (w[u] != 0.f) {
                    wsum += w[u];
                    acc.x = fmaf(w[u], o[u].x, acc.x);
                    acc.y = fmaf(w[u], o[u].y, acc.y);
                    acc.z = fmaf(w[u], o[u].z, acc.z);
                    acc.w = fmaf(w[u], o[u].w, acc.w);
                }
            }
        }
    }
    const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    if constexpr (OD == MOSKA_BF16) {
        uint2 v;
        v.x = f32_to_bf16_bits(acc.x) | (f32_to_bf16_bits(acc.y) << 16);
        v.y = f32_to_bf16_bits(acc.z) | (f32_to_bf16_bits(acc.w) << 16);
        *(uint2 *)((uint16_t *)O + r * D + 4 * t) = v;
    } else {
        *(float4 *)((float *)O + r * D + 4 * t) = acc;
    }
    if (LSE && t == 0) LSE[r] = wsum > 0.f ? m + logf(wsum) : -INFINITY;
}

// The same combination for many partial slots (P in the hundreds: a quarter of thousands of chunks):
// a workgroup of 256 threads per row, the slots dealt round-robin to its 256/(D/4) thread groups,
// whose partial (weight sum, weighted O) are added through LDS.  D/4 must divide 256.
template <int OD>
__global__ __launch_bounds__(256) void merge_wide_kernel(const float *__restrict__ part_O,
                                                          const float *__restrict__ part_LSE, void *__restrict__ O,
                                                          float *__restrict__ LSE, int P, int D) {
    __shared__ float red[256 * 4 + 64];
    const int tpr = D / 4, ng = 256 / tpr;                  // threads per slot, slot groups
    const int t = threadIdx.x % tpr, g = threadIdx.x / tpr;
    const int64_t r = blockIdx.x;
    const float *lse = part_LSE + r * P;
    // row maximum: every thread a strided share of the slots, then waves, then the block
    float m = -INFINITY;
    for (int j = threadIdx.x; j < P; j += 256) m = fmaxf(m, lse[j]);
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1) m = fmaxf(m, __shfl_xor(m, w));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float wsum = 0.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    if (m != -INFINITY) {
        const float *po = part_O + r * P * D + 4 * t;
        for (int j0 = g; j0 < P; j0 += 4 * ng) {            // four slots of the group per round, loads issued together
            float4 o[4];
            float w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = min(j0 + u * ng, P - 1);
                o[u] = *(const float4 *)(po + (int64_t)j * D);
                const float lj = lse[j];
                w[u] = (j0 + u * ng < P && lj != -INFINITY) ? expf(lj - m) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (w[u] != 0.f) {
                    wsum += w[u];
                    acc.x = fmaf(w[u], o[u].x, acc.x);
                    acc.y = fmaf(w[u], o[u].y, acc.y);
                    acc.z = fmaf(w[u], o[u].z, acc.z);
                    acc.w = fmaf(w[u], o[u].w, acc.w);
                }
            }
        }
    }
    // add the groups' sums in a fixed order (deterministic)
    *(float4 *)(red + 4 * threadIdx.x) = acc;
    if (t == 0) red[1024 + g] = wsum;
    __syncthreads();
    if (g != 0) return;
    for (int gg = 1; gg < ng; ++gg) {
        const float4 o = *(const float4 *)(red + 4 * (gg * tpr + t));
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
        wsum += red[1024 + gg];
    }
    const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    if constexpr (OD == MOSKA_BF16) {
        uint2 v;
        v.x = f32_to_bf16_bits(acc.x) | (f32_to_bf16_bits(acc.y) << 16);
        v.y = f32_to_bf16_bits(acc.z) | (f32_to_bf16_bits(acc.w) << 16);
        *(uint2 *)((uint16_t *)O + r * D + 4 * t) = v;
    } else {
        *(float4 *)((float *)O + r * D + 4 * t) = acc;
    }
    if (LSE && t == 0) LSE[r] = wsum > 0.f ? m + logf(wsum) : -INFINITY;
}

}  // namespace

int launch_merge(const moska_problem_t &p, const float *part_O, const float *part_LSE, void *O, float *LSE,
                 hipStream_t s) {
    const int64_t rows = (int64_t)p.B * p.Hq;
    if (p.k + 1 >= 64 && 256 % (p.D / 4) == 0 && 256 / (p.D / 4) <= 64) {   // many slots: a workgroup per row
        auto wide = p.q_dtype == MOSKA_BF16 ? merge_wide_kernel<MOSKA_BF16> : merge_wide_kernel<MOSKA_F32>;
        hipLaunchKernelGGL(wide, dim3((unsigned)rows), dim3(256), 0, s, part_O, part_LSE, O, LSE, p.k + 1, p.D);
        return hip_status(hipGetLastError());
    }
    const int rpb = 256 / (p.D / 4);
    const unsigned grid = (unsigned)((rows + rpb - 1) / rpb);
    auto kern = p.q_dtype == MOSKA_BF16 ? merge_kernel<MOSKA_BF16> : merge_kernel<MOSKA_F32>;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, s, part_O, part_LSE, O, LSE, rows, p.k + 1, p.D);
    return hip_status(hipGetLastError());
}

}  // namespace moska
