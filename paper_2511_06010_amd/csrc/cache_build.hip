// Offline construction of the shared KV store (paper Sec. III-A: pre-computed shared caches;
// Sec. III-B: precomputed chunk embeddings).  Two streaming kernels, one workgroup per
// (chunk, KV head) block, both bound by HBM traffic on the block they read:
//   chunk_embeddings  E[h,c,:] = mean over the block's L stored keys (fp64 accumulation)
//   quantize_fp8      per-block scale = amax/448 and the block re-expressed in OCP e4m3fn
#include "moska_internal.h"

namespace moska {
namespace {

template <int DT> constexpr int elem_bytes() { return DT == MOSKA_F32 ? 4 : DT == MOSKA_BF16 ? 2 : 1; }

// the n = 16/elem_bytes values of one 16-byte unit as floats
template <int DT>
__device__ __forceinline__ void unpack16(const uint4 &u, float *v) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
    if constexpr (DT == MOSKA_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(w[i]);
    } else if constexpr (DT == MOSKA_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    } else {
        typedef __attribute__((ext_vector_type(2))) float f32x2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {                       // v_cvt_pk_f32_fp8: two bytes per instruction, exact
            const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
            v[4 * i] = lo[0]; v[4 * i + 1] = lo[1]; v[4 * i + 2] = hi[0]; v[4 * i + 3] = hi[1];
        }
    }
}

// Thread (r, u): unit u of the key row (16 bytes = N dims), token rows r, r+R, ...; the R partial
// sums of every dim are added through LDS.
template <int KVD, int QD>
__global__ __launch_bounds__(256) void chunk_embeddings_kernel(const void *__restrict__ Ks,
                                                                const float *__restrict__ scale_k,
                                                                void *__restrict__ E, int Hkv, int C, int L, int D) {
    constexpr int N = 16 / elem_bytes<KVD>();
    extern __shared__ double red[];                         // [R][D]
    const int upr = D / N, R = 256 / upr;                   // units per row, token rows per pass
    const int c = blockIdx.x / Hkv, h = blockIdx.x - c * Hkv;
    const int r = threadIdx.x / upr, u = threadIdx.x - r * upr;
    const uint4 *base = (const uint4 *)((const char *)Ks + ((int64_t)c * Hkv + h) * L * D * elem_bytes<KVD>());
    double acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.0;
    if (r < R) {
        if constexpr (KVD == MOSKA_FP8_E4M3) {
            // e4m3 values are multiples of 2^-9 of magnitude <= 448: 32 of them add up exactly in f32
            // (23 bits), so the fp64 accumulator is touched once per 32 rows; every sum here is exact
            // in any order, and so is the reference's.
            for (int t0 = r; t0 < L; t0 += 32 * R) {
                float part[N];
#pragma unroll
                for (int i = 0; i < N; ++i) part[i] = 0.f;
                for (int t = t0; t < min(L, t0 + 32 * R); t += R) {
                    float v[N];
                    unpack16<KVD>(base[(int64_t)t * upr + u], v);
#pragma unroll
                    for (int i = 0; i < N; ++i) part[i] += v[i];
                }
#pragma unroll
                for (int i = 0; i < N; ++i) acc[i] += (double)part[i];
            }
        } else {
            for (int t = r; t < L; t += R) {
                float v[N];
                unpack16<KVD>(base[(int64_t)t * upr + u], v);
#pragma unroll
                for (int i = 0; i < N; ++i) acc[i] += (double)v[i];
            }
        }
#pragma unroll
        for (int i = 0; i < N; ++i) red[r * D + u * N + i] = acc[i];
    }
    __syncthreads();
    const double mul = (scale_k ? (double)scale_k[c * Hkv + h] : 1.0);
    for (int d = threadIdx.x; d < D; d += 256) {
        double s = 0.0;
        for (int rr = 0; rr < R; ++rr) s += red[rr * D + d];
        const float m = (float)(mul * s / (double)L);
        const int64_t o = ((int64_t)h * C + c) * D + d;
        if constexpr (QD == MOSKA_F32) ((float *)E)[o] = m;
        else ((uint16_t *)E)[o] = (uint16_t)f32_to_bf16_bits(m);
    }
}

__device__ __forceinline__ float block_max(float v, float *tmp) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m));
    if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = v;
    __syncthreads();
    v = fmaxf(fmaxf(tmp[0], tmp[1]), fmaxf(tmp[2], tmp[3]));
    __syncthreads();
    return v;
}

// X: bf16 block of n16 16-byte units; two passes over it (the second one hits L2)
__global__ __launch_bounds__(256) void quantize_fp8_kernel(const void *__restrict__ X, void *__restrict__ X8,
                                                            float *__restrict__ scale, int64_t units_per_block) {
    __shared__ float tmp[4];
    const uint4 *src = (const uint4 *)X + (int64_t)blockIdx.x * units_per_block;
    uint2 *dst = (uint2 *)X8 + (int64_t)blockIdx.x * units_per_block;
    float amax = 0.f;
    for (int64_t i = threadIdx.x; i < units_per_block; i += 256) {
        float v[8];
        unpack16<MOSKA_BF16>(src[i], v);
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(v[j]));
    }
    amax = block_max(amax, tmp);
    const float sc = fmaxf(amax / 448.0f, 1e-30f);
    if (threadIdx.x == 0) scale[blockIdx.x] = sc;
    for (int64_t i = threadIdx.x; i < units_per_block; i += 256) {
        float v[8];
        unpack16<MOSKA_BF16>(src[i], v);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = fminf(fmaxf(v[j] / sc, -448.f), 448.f);
        int lo = 0, hi = 0;                               // v_cvt_pk_fp8_f32: round to nearest even
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], lo, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], lo, true);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], hi, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], hi, true);
        dst[i] = uint2{(uint32_t)lo, (uint32_t)hi};
    }
}

}  // namespace

int launch_chunk_embeddings(const moska_problem_t &p, const void *Ks, const float *scale_k, void *E, hipStream_t s) {
    const int kvd = p.shared_kv_dtype, esz = kvd == MOSKA_F32 ? 4 : kvd == MOSKA_BF16 ? 2 : 1;
    const int upr = p.D * esz / 16;
    if (upr < 1 || upr > 256 || (p.D * esz) % 16) return MOSKA_ERR_UNSUPPORTED;
    const int R = 256 / upr;
    const size_t lds = (size_t)R * p.D * sizeof(double);
    const unsigned grid = (unsigned)(p.C * p.Hkv);
    void (*kern)(const void *, const float *, void *, int, int, int, int) = nullptr;
    if (kvd == MOSKA_F32) kern = chunk_embeddings_kernel<MOSKA_F32, MOSKA_F32>;
    else if (kvd == MOSKA_BF16) kern = chunk_embeddings_kernel<MOSKA_BF16, MOSKA_BF16>;
    else kern = chunk_embeddings_kernel<MOSKA_FP8_E4M3, MOSKA_BF16>;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return MOSKA_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, Ks, scale_k, E, p.Hkv, p.C, p.L, p.D);
    return hip_status(hipGetLastError());
}

int launch_quantize_fp8(const moska_problem_t &p, const void *X, void *X8, float *scale, hipStream_t s) {
    if ((p.L * p.D) % 8) return MOSKA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(quantize_fp8_kernel, dim3(p.C * p.Hkv), dim3(256), 0, s, X, X8, scale,
                       (int64_t)p.L * p.D / 8);
    return hip_status(hipGetLastError());
}

}  // namespace moska
