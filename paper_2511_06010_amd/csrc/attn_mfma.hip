// MFMA Unique KV Attention launcher and the dispatch of the MFMA Shared KV Attention variants.
#include <cstdlib>

#include "attn_mfma.h"

namespace moska {

int launch_shared_mfma_bf16(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s);
int launch_shared_mfma_fp8(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s);

namespace {
using mfma::HD;

// Log-sum-exp combination of the ns slices of every row of a split attention.  Row r of the split
// workspace belongs to query row r / per_row and partial slot slot0 + r % per_row (shared:
// per_row = k, slot0 = 0; unique: per_row = 1, slot0 = k).  One thread per (row, 4 dims).
__global__ __launch_bounds__(256) void split_combine_kernel(const float *__restrict__ split_O,
                                                            const float *__restrict__ split_LSE, int ns, int64_t rows,
                                                            int k, int per_row, int slot0, float *__restrict__ part_O,
                                                            float *__restrict__ part_LSE) {
    const int t = threadIdx.x & 31;                         // 32 threads x 4 dims = HD
    const int64_t r = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
    if (r >= rows) return;
    const float *lse = split_LSE + r * ns;
    float m = -INFINITY;
    for (int s = 0; s < ns; ++s) m = fmaxf(m, lse[s]);
    float wsum = 0.f;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    if (m != -INFINITY) {
        for (int s = 0; s < ns; ++s) {
            const float ls = lse[s];
            if (ls == -INFINITY) continue;
            const float w = expf(ls - m);
            wsum += w;
            const float4 o = *(const float4 *)(split_O + (r * ns + s) * HD + 4 * t);
            acc.x = fmaf(w, o.x, acc.x); acc.y = fmaf(w, o.y, acc.y);
            acc.z = fmaf(w, o.z, acc.z); acc.w = fmaf(w, o.w, acc.w);
        }
    }
    const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    const int64_t o = (r / per_row) * (k + 1) + slot0 + r % per_row;
    *(float4 *)(part_O + o * HD + 4 * t) = acc;
    if (t == 0) part_LSE[o] = wsum > 0.f ? m + logf(wsum) : -INFINITY;
}

int launch_split_combine(const float *split_O, const float *split_LSE, int ns, int64_t rows, int k, int per_row,
                         int slot0, float *part_O, float *part_LSE, hipStream_t s) {
    hipLaunchKernelGGL(split_combine_kernel, dim3((unsigned)((rows + 7) / 8)), dim3(256), 0, s, split_O, split_LSE, ns,
                       rows, k, per_row, slot0, part_O, part_LSE);
    return hip_status(hipGetLastError());
}

}  // namespace

int launch_shared_mfma(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    if (int rc = p.shared_kv_dtype == MOSKA_FP8_E4M3 ? launch_shared_mfma_fp8(p, a, pl, s)
                                                     : launch_shared_mfma_bf16(p, a, pl, s))
        return rc;
    if (a.nsplit > 1)
        return launch_split_combine(a.split_O, a.split_LSE, a.nsplit, (int64_t)p.B * p.Hq * p.k, p.k, p.k, 0,
                                    a.part_O, a.part_LSE, s);
    return MOSKA_OK;
}

int launch_unique_mfma(const moska_problem_t &p, const UniqueArgs &a, hipStream_t s) {
    using namespace mfma;
    // 16, 32 or 64 query rows per workgroup; 4 waves split the keys, non-temporal loads, one key tile
    // in flight per wave (two for the 64-row kernel, which runs one wave per SIMD)
    int T = q_len(p);
    const int R = T * (p.Hq / p.Hkv);                          // query rows per (request, KV head)
    const int NR = R <= 16 ? 1 : R <= 32 ? 2 : 4;
    // [split run?][row blocks]: the slices of a split run are written write-back for the combine kernel
    static const void *const table[2][3] = {
        {(const void *)unique_mfma_kernel<1, 4, 2, 1, false>, (const void *)unique_mfma_kernel<2, 4, 2, 1, false>,
         (const void *)unique_mfma_kernel<4, 4, 2, 2, false>},
        {(const void *)unique_mfma_kernel<1, 4, 2, 1, true>, (const void *)unique_mfma_kernel<2, 4, 2, 1, true>,
         (const void *)unique_mfma_kernel<4, 4, 2, 2, true>}};
    const void *kernel = table[a.nsplit > 1][NR == 1 ? 0 : NR == 2 ? 1 : 2];
    const int gt = (R + 16 * NR - 1) / (16 * NR);
    const unsigned grid = (unsigned)((int64_t)p.B * p.Hkv * gt * a.nsplit);
    UniqueArgs args = a;
    int Hq = p.Hq, Hkv = p.Hkv, U = p.U_max, k = p.k;
    float scale = p.scale;
    void *kargs[] = {&args, &Hq, &Hkv, &U, &k, &scale, &T};
    if (hipLaunchKernel(kernel, dim3(grid), dim3(256), kargs, 0, s) != hipSuccess) return MOSKA_ERR_HIP;
    if (a.nsplit > 1)
        return launch_split_combine(a.split_O, a.split_LSE, a.nsplit, (int64_t)p.B * T * p.Hq, p.k, 1, p.k, a.part_O,
                                    a.part_LSE, s);
    return MOSKA_OK;
}

}  // namespace moska
