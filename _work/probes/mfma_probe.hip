// mfma_probe: two stand-alone measurements behind the design of the compute-bound shared-attention
// tiles (no input data, no library call; it only includes the kernels' own inner-loop helpers).
//   (a) Do matrix-core and vector-ALU instructions of one SIMD overlap?  Eight waves per workgroup,
//       one workgroup per compute unit (wave w runs on SIMD w % 4): waves 0-3 issue MFMAs, waves 4-7
//       vector FMAs, alone and together, and one wave interleaves both.
//   (b) How fast is the inner loop of the 256-row tile (scores, online softmax, P V; operands read
//       from LDS) with nothing else around it -- no global loads, no stage writes, no tile prologue?
// Usage: mfma_probe
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include "attn_mfma_lds.h"
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
using namespace moska;
using namespace moska::mfma;

// ---- (a) -----------------------------------------------------------------------------------------
// mode per wave: bit w of mfma_mask -> 8 MFMAs per iteration, bit w of valu_mask -> NFMA FMAs per
// iteration; BOTH: the MFMA waves interleave the FMAs between their MFMAs.
template <int NFMA, bool BOTH>
__global__ __launch_bounds__(512, 2) void overlap_kernel(float *out, int iters, unsigned mfma_mask, unsigned valu_mask) {
    __shared__ float pad[20 * 1024];                       // 80 KB: one workgroup per compute unit
    const int wave = threadIdx.x >> 6;
    f32x4 acc[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    float v[8];
    for (int i = 0; i < 8; ++i) v[i] = threadIdx.x * 0.001f + i;
    uint32_t a[4], b[4];
    for (int i = 0; i < 4; ++i) { a[i] = 0x3c003c00u + threadIdx.x; b[i] = 0x3c003c00u + i; }
    if ((mfma_mask >> wave) & 1) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                acc[u & 3] = mfma16(a, b, acc[u & 3]);
                if (BOTH) {
#pragma unroll
                    for (int w = 0; w < NFMA / 8; ++w) v[(u + w) & 7] = __builtin_fmaf(v[(u + w) & 7], 1.0001f, 0.5f);
                }
            }
        }
    } else if ((valu_mask >> wave) & 1) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < NFMA; ++u) v[u & 7] = __builtin_fmaf(v[u & 7], 1.0001f, 0.5f);
        }
    }
    float r = 0;
    for (int i = 0; i < 4; ++i) r += acc[i][0] + acc[i][1];
    for (int i = 0; i < 8; ++i) r += v[i];
    if (r == 123.456f) out[threadIdx.x] = r + pad[threadIdx.x];
}

template <int NFMA, bool BOTH> float run_overlap(float *out, unsigned mm, unsigned vm, int iters) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    hipLaunchKernelGGL((overlap_kernel<NFMA, BOTH>), dim3(256), dim3(512), 0, 0, out, iters, mm, vm);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((overlap_kernel<NFMA, BOTH>), dim3(256), dim3(512), 0, 0, out, iters, mm, vm);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    return ms;
}

// ---- (b) -----------------------------------------------------------------------------------------
// NWV waves of 16*NR rows each run `stages` 64-key stages out of two LDS buffers filled once.
template <int NR, int NWV>
__global__ __launch_bounds__(NWV * 64, 2) void loop_kernel(float *out, int stages) {
    __shared__ uint4 smem[lds_units<64>()];
    constexpr int SU = 64 * 16;
    uint4 *ldsK = smem, *ldsV = smem + 2 * SU;
    const int tid = threadIdx.x, lane = tid & 63, q = lane >> 4, x = lane & 15;
    for (int i = tid; i < 4 * SU; i += NWV * 64) {          // small bf16 values
        const uint32_t w = 0x3c003c00u + ((i * 2654435761u) & 0x007f007fu);
        smem[i] = uint4{w, w ^ 0x80000000u, w, w ^ 0x00008000u};
    }
    __syncthreads();
    uint32_t qf[NR][4][4];
    for (int rb = 0; rb < NR; ++rb)
        for (int kb = 0; kb < 4; ++kb)
            for (int i = 0; i < 4; ++i) qf[rb][kb][i] = 0x3c003c00u + ((lane + 7 * kb + i + rb) & 0x7f);
    WaveState<NR> st;
    for (int rb = 0; rb < NR; ++rb) {
        st.m[rb] = -INFINITY;
        st.l[rb] = 0.f;
        for (int e = 0; e < 8; ++e) st.o[rb][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int L = stages * 64;
    for (int t = 0; t < stages; ++t) {
        const int cur = t & 1;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            f32x4 s[NR][2];
            uint32_t pf[NR][4];
            qk_from_lds<NR>(s, qf, ldsK + cur * SU + sub * 512, q, x);
            softmax_tile<NR, false>(st, s, pf, 64 * t + 32 * sub, L, 0.01f, q);
            pv_from_lds<NR>(st, ldsV + cur * SU + sub * 512, pf, lane);
        }
    }
    float r = 0.f;
    for (int rb = 0; rb < NR; ++rb) {
        r += st.l[rb] + st.m[rb];
        for (int e = 0; e < 8; ++e) r += st.o[rb][e][0] + st.o[rb][e][3];
    }
    if (r == 123.456f) out[tid] = r;
}

template <int NR, int NWV> void run_loop(float *out, const char *name, int wgs_per_cu) {
    const int stages = 2000, grid = 256 * wgs_per_cu;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    hipLaunchKernelGGL((loop_kernel<NR, NWV>), dim3(grid), dim3(NWV * 64), 0, 0, out, 10);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((loop_kernel<NR, NWV>), dim3(grid), dim3(NWV * 64), 0, 0, out, stages);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double rows = 16.0 * NR * NWV * grid, flops = 4.0 * 128 * rows * stages * 64;
    printf("%-64s: %.3f ms  %.0f TFLOP/s (%.1f %% of 2500)\n", name, ms, flops / ms / 1e9, flops / ms / 1e9 / 25.0);
}

int main() {
    float *out;
    CK(hipMalloc(&out, 8192));
    const int iters = 20000;
    printf("(a) per iteration: 8 x v_mfma_f32_16x16x32_bf16 per MFMA wave, 32 x v_fma_f32 per vector-ALU wave; %d iterations\n", iters);
    printf("waves 0-3 MFMA, 4-7 idle                      : %.3f ms\n", run_overlap<32, false>(out, 0x0F, 0x00, iters));
    printf("waves 0-7 MFMA (two per SIMD)                 : %.3f ms\n", run_overlap<32, false>(out, 0xFF, 0x00, iters));
    printf("waves 0-3 idle, 4-7 FMA                       : %.3f ms\n", run_overlap<32, false>(out, 0x00, 0xF0, iters));
    printf("waves 0-3 MFMA, 4-7 FMA (one of each per SIMD): %.3f ms\n", run_overlap<32, false>(out, 0x0F, 0xF0, iters));
    printf("waves 0-3 MFMA and FMA interleaved, 4-7 idle  : %.3f ms\n", run_overlap<32, true>(out, 0x0F, 0x00, iters));
    printf("(b) inner loop of the LDS tiles alone (head size 128, 64-key stages out of LDS, 2000 stages)\n");
    run_loop<2, 4>(out, "4 waves x 32 rows, one workgroup per CU (one wave per SIMD)", 1);
    run_loop<2, 8>(out, "8 waves x 32 rows, one workgroup per CU (two waves per SIMD)", 1);
    run_loop<2, 4>(out, "4 waves x 32 rows, two workgroups per CU (two waves per SIMD)", 2);
    run_loop<1, 8>(out, "8 waves x 16 rows, two workgroups per CU (four waves per SIMD)", 2);
    return 0;
}
