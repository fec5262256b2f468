// moska_route: chunk scoring and top-k selection (paper Sec. III-B).
//
// Scoring is a dense fp64 contraction per KV head, S_h[B x C] = Qsum_h[B x D] * E_h^T[D x C], and runs
// on the fp64 matrix cores (v_mfma_f64_16x16x4_f64): products of f32 or bf16 inputs are exact in
// fp64, so the scores agree with an fp64 reference to the rounding order of the sums.  A wave
// owns 16 requests of one head; the 16 x D block of group-summed queries stays in its registers as
// the A operands while it walks over 16-chunk tiles of E, whose rows it reads with 16-byte loads
// (the contraction index is permuted so that what a lane loads is what it feeds).  Scores leave
// as order-preserving 64-bit keys in the workspace.
//
// Selection: one wave per (request, KV head) extracts the k best in k rounds of "largest key of the
// wave, lowest chunk id among its holders".  Up to 1024 chunks the keys stay in registers (lane l holds
// chunks l, l+64, ...) and the wave-wide maximum / minimum run on the vector ALU (DPP permutes, then
// v_permlane16_swap / v_permlane32_swap); above that the keys sit in LDS and only a round's winner
// rescans its chunks -- unless k is large too (the paper's 75 % sparsity keeps a quarter of thousands
// of chunks): then a workgroup sorts the row's keys with a bitonic network and writes the first k.
//
// Head sizes other than 64/128/256 take a vector-ALU scoring kernel (one chunk row per lane).
#include "moska_internal.h"

namespace moska {
namespace {

typedef __attribute__((ext_vector_type(4))) double f64x4;

__device__ __forceinline__ uint64_t order_key(double s) {
    s = s + 0.0;                                   // -0.0 and +0.0 must tie
    uint64_t u = (uint64_t)__double_as_longlong(s);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double key_to_score(uint64_t k) {
    uint64_t u = (k >> 63) ? (k & 0x7FFFFFFFFFFFFFFFull) : ~k;
    return __longlong_as_double((long long)u);
}

// elements of a 16-byte load
template <int QD> constexpr int epl() { return QD == MOSKA_BF16 ? 8 : 4; }

template <int QD>
__device__ __forceinline__ void widen16(const uint4 &v, double (&out)[epl<QD>()]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    if constexpr (QD == MOSKA_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = (double)__uint_as_float(w[i] << 16);
            out[2 * i + 1] = (double)__uint_as_float(w[i] & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = (double)__uint_as_float(w[i]);
    }
}

// Scores of 16 requests x (a range of) 16-chunk tiles of one head, on the fp64 matrix cores.
// D = NBLK * 4 * epl.  MFMA operands: lane (g = lane/16, x = lane%16) holds A[x][g], B[g][x] and, in
// result register i, C[4i + g][x].  Step (blk, j) of the contraction takes dim blk*4*epl + g*epl + j from lane group
// g, for A and B alike, so a lane's 16-byte load of a row supplies epl consecutive steps.
template <int QD, int NBLK>
__global__ __launch_bounds__(256) void route_score_kernel(const void *__restrict__ Q, const void *__restrict__ E,
                                                           uint64_t *__restrict__ keys, int B, int Hq, int Hkv, int C,
                                                           int btiles, int csplit, int ctiles) {
    constexpr int EPL = epl<QD>(), D = NBLK * 4 * EPL, ESZ = QD == MOSKA_BF16 ? 2 : 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + wave;
    const int cs = w % csplit, bt = (w / csplit) % btiles, h = w / (csplit * btiles);
    if (h >= Hkv) return;
    const int g = lane >> 4, x = lane & 15, G = Hq / Hkv;
    const int per = (ctiles + csplit - 1) / csplit;
    const int ct0 = cs * per, ct1 = min(ctiles, ct0 + per);
    if (ct0 >= ct1) return;

    // A operands: the group-summed query of request bt*16 + x (rows past B repeat the last one)
    double a[NBLK * EPL];
#pragma unroll
    for (int i = 0; i < NBLK * EPL; ++i) a[i] = 0.0;
    {
        const int b = min(bt * 16 + x, B - 1);
        const char *qrow = (const char *)Q + ((int64_t)b * Hq + (int64_t)h * G) * D * ESZ + g * 16;
        for (int gh = 0; gh < G; ++gh) {
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
                double t[EPL];
                widen16<QD>(*(const uint4 *)(qrow + ((int64_t)gh * D + blk * 4 * EPL) * ESZ), t);
#pragma unroll
                for (int j = 0; j < EPL; ++j) a[blk * EPL + j] += t[j];
            }
        }
    }

    const char *ebase = (const char *)E + (int64_t)h * C * D * ESZ + g * 16;
    auto load_tile = [&](uint4 (&e)[NBLK], int ct) {
        const int c = min(ct * 16 + x, C - 1);                 // columns past C repeat the last chunk
        const char *row = ebase + (int64_t)c * D * ESZ;
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) e[blk] = *(const uint4 *)(row + blk * 4 * EPL * ESZ);
    };
    uint4 e[NBLK], en[NBLK];
    load_tile(e, ct0);
    for (int ct = ct0; ct < ct1; ++ct) {
        if (ct + 1 < ct1) load_tile(en, ct + 1);
        f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            double t[EPL];
            widen16<QD>(e[blk], t);
#pragma unroll
            for (int j = 0; j < EPL; ++j) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[blk * EPL + j], t[j], acc, 0, 0, 0);
        }
        const int c = ct * 16 + x;
        if (c < C) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int b = bt * 16 + 4 * i + g;
                if (b < B) keys[((int64_t)b * Hkv + h) * C + c] = order_key(acc[i]);
            }
        }
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) e[blk] = en[blk];
    }
}

// Wave-wide reductions that leave the result in every lane, on the vector ALU alone: two quad
// permutes, two mirrors inside a row of 16 lanes (DPP), then the xor-16 / xor-32 pairs through
// v_permlane16_swap / v_permlane32_swap.  (Six ds_bpermute rounds cost several times as much.)
template <int CTRL> __device__ __forceinline__ uint32_t dpp(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL> __device__ __forceinline__ uint64_t dpp64(uint64_t v) {
    return ((uint64_t)dpp<CTRL>((uint32_t)(v >> 32)) << 32) | dpp<CTRL>((uint32_t)v);
}
__device__ __forceinline__ uint64_t max_u64(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
    v = max_u64(v, dpp64<0xB1>(v));                        // quad_perm [1,0,3,2]
    v = max_u64(v, dpp64<0x4E>(v));                        // quad_perm [2,3,0,1]
    v = max_u64(v, dpp64<0x141>(v));                       // row_half_mirror
    v = max_u64(v, dpp64<0x140>(v));                       // row_mirror
    const uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    auto l16 = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    auto h16 = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    v = max_u64(((uint64_t)h16[0] << 32) | l16[0], ((uint64_t)h16[1] << 32) | l16[1]);
    const uint32_t lo2 = (uint32_t)v, hi2 = (uint32_t)(v >> 32);
    auto l32 = __builtin_amdgcn_permlane32_swap(lo2, lo2, false, false);
    auto h32 = __builtin_amdgcn_permlane32_swap(hi2, hi2, false, false);
    return max_u64(((uint64_t)h32[0] << 32) | l32[0], ((uint64_t)h32[1] << 32) | l32[1]);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = min(v, dpp<0xB1>(v));
    v = min(v, dpp<0x4E>(v));
    v = min(v, dpp<0x141>(v));
    v = min(v, dpp<0x140>(v));
    auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = min(a[0], a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return min(b[0], b[1]);
}

// The k best of the wave's C keys (in LDS), written to ids/scores of row o = (b*Hkv + h).
// Each lane remembers the best of its own chunks; a round takes the largest key of the wave and,
// among the lanes that hold it, the lowest chunk id; only the round's winner rescans.
__device__ __forceinline__ void select_topk(uint64_t *keys, int C, int k, int lane, bool active, int64_t o,
                                            int32_t *__restrict__ ids, float *__restrict__ scores) {
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
        const uint64_t wk = wave_max_u64(bk);
        const int wc = (int)wave_min_u32(bk == wk ? (uint32_t)bc : 0x7FFFFFFFu);
        if (lane == (wc & (kWave - 1))) {
            keys[wc] = 0;
            rescan(bk, bc);
        }
        if (active && lane == 0) {
            ids[o * k + t] = wc;
            if (scores) scores[o * k + t] = (float)key_to_score(wk);
        }
    }
}

// One wave per (request, KV head): keys from the workspace into LDS, then the selection.
__global__ __launch_bounds__(256) void route_select_kernel(const uint64_t *__restrict__ gkeys, int32_t *__restrict__ ids,
                                                            float *__restrict__ scores, int64_t rows, int C, int k,
                                                            int W) {
    extern __shared__ double smem[];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    int64_t r = (int64_t)blockIdx.x * W + wave;    // r = b*Hkv + h
    const bool active = r < rows;
    if (!active) r = rows - 1;                     // compute redundantly, write nothing
    uint64_t *keys = (uint64_t *)smem + (size_t)wave * C;
    for (int c = lane; c < C; c += kWave) keys[c] = gkeys[r * C + c];
    __syncthreads();
    select_topk(keys, C, k, lane, active, r, ids, scores);
}

// The same selection with the keys in registers (up to 64*KPL chunks: lane l holds chunks l, l+64, ...):
// no LDS, no divergent rescans -- every lane re-derives its best key from its KPL registers each round.
template <int KPL>
__global__ __launch_bounds__(256) void route_select_reg_kernel(const uint64_t *__restrict__ gkeys,
                                                                int32_t *__restrict__ ids, float *__restrict__ scores,
                                                                int64_t rows, int C, int k) {
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int64_t r = (int64_t)blockIdx.x * 4 + wave;      // r = b*Hkv + h
    if (r >= rows) return;
    uint64_t key[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) {
        const int c = lane + kWave * i;
        key[i] = c < C ? gkeys[r * C + c] : 0;             // 0 is below every real key
    }
    for (int t = 0; t < k; ++t) {
        uint64_t bk = key[0];
        int bi = 0;
#pragma unroll
        for (int i = 1; i < KPL; ++i) {
            if (key[i] > bk) { bk = key[i]; bi = i; }      // equal keys: the lower chunk id stays
        }
        const uint64_t wk = wave_max_u64(bk);
        const int wc = (int)wave_min_u32(bk == wk ? (uint32_t)(lane + kWave * bi) : 0x7FFFFFFFu);
#pragma unroll
        for (int i = 0; i < KPL; ++i) {
            if (wc == lane + kWave * i) key[i] = 0;
        }
        if (lane == 0) {
            ids[r * k + t] = wc;
            if (scores) scores[r * k + t] = (float)key_to_score(wk);
        }
    }
}

// Selection by sorting, for many chunks AND a large k (the k-round selections above cost k wave-wide
// reductions per row): one workgroup of 256 threads sorts the row's N = 256*EPT (key, chunk) pairs,
// C padded with keys below every real one, into the order (key descending, chunk ascending) with a
// bitonic network and writes the first k.  Thread t owns elements t*EPT .. t*EPT+EPT-1 in
// registers: compare-exchange steps with a stride below EPT stay inside the thread; for the
// others the threads swap elements through LDS (element e of thread t at [e][t]: conflict free).
template <int EPT>
__global__ __launch_bounds__(256) void route_sort_kernel(const uint64_t *__restrict__ gkeys, int32_t *__restrict__ ids,
                                                          float *__restrict__ scores, int C, int k) {
    constexpr int N = 256 * EPT;
    __shared__ uint64_t xkey[EPT][256];
    __shared__ int32_t xid[EPT][256];
    const int t = threadIdx.x;
    const int64_t r = blockIdx.x;                           // r = b*Hkv + h
    uint64_t key[EPT];
    int32_t id[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int c = t * EPT + e;
        key[e] = c < C ? gkeys[r * C + c] : 0;              // 0 is below every real key
        id[e] = c < C ? c : 0x7FFFFFFF;
    }
    // a goes before b
    auto before = [](uint64_t ka, int32_t ia, uint64_t kb, int32_t ib) { return ka > kb || (ka == kb && ia < ib); };
#pragma unroll
    for (int size = 2; size <= N; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride < EPT) {
#pragma unroll
                for (int e = 0; e < EPT; ++e) {
                    if (e & stride) continue;               // the lower element of each pair does the exchange
                    const int f = e | stride;
                    const bool up = ((t * EPT + e) & size) == 0;          // this block is sorted best first
                    const bool swap = before(key[f], id[f], key[e], id[e]) == up;
                    const uint64_t ke = key[e], kf = key[f];
                    const int32_t ie = id[e], jf = id[f];
                    key[e] = swap ? kf : ke; key[f] = swap ? ke : kf;
                    id[e] = swap ? jf : ie;  id[f] = swap ? ie : jf;
                }
            } else {
                __syncthreads();                            // the previous exchange has been read
#pragma unroll
                for (int e = 0; e < EPT; ++e) {
                    xkey[e][t] = key[e];
                    xid[e][t] = id[e];
                }
                __syncthreads();
                const int pt = t ^ (stride / EPT);          // the thread that owns the partners
                const bool lower = (t & (stride / EPT)) == 0;
#pragma unroll
                for (int e = 0; e < EPT; ++e) {
                    const bool up = ((t * EPT + e) & size) == 0;
                    const uint64_t kp = xkey[e][pt];
                    const int32_t ip = xid[e][pt];
                    // keep the better of the two in the lower position of a best-first block, the worse otherwise
                    const bool take = before(kp, ip, key[e], id[e]) == (up == lower);
                    key[e] = take ? kp : key[e];
                    id[e] = take ? ip : id[e];
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int g = t * EPT + e;
        if (g < k) {
            ids[r * k + g] = id[e];
            if (scores) scores[r * k + g] = (float)key_to_score(key[e]);
        }
    }
}

// Vector-ALU scoring for the other head sizes: one wave per (request, KV head), lane l scores
// chunks l, l+64, ... with fp64 FMAs, then the same selection.
template <int QD>
__global__ __launch_bounds__(256) void route_lane_kernel(const void *__restrict__ Q, const void *__restrict__ E,
                                                          int32_t *__restrict__ ids, float *__restrict__ scores,
                                                          int B, int Hq, int Hkv, int D, int C, int k, int W) {
    extern __shared__ double smem[];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int64_t rows = (int64_t)B * Hkv;
    int64_t r = (int64_t)blockIdx.x * W + wave;    // r = h*B + b: the waves of a block share E[h]
    const bool active = r < rows;
    if (!active) r = rows - 1;
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
        for (int d = 0; d < D; ++d) a = fma(qs[d], (double)load_f32<QD>(E, base + d), a);
        keys[c] = order_key(a);
    }
    __syncthreads();
    select_topk(keys, C, k, lane, active, (int64_t)b * Hkv + h, ids, scores);
}

template <typename K>
int raise_lds_limit(K kern, size_t lds) {
    if (lds <= 48 * 1024) return MOSKA_OK;
    return hip_status(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
}

template <int QD>
const void *score_kernel_for(int D) {
    constexpr int U = 4 * epl<QD>();
    switch (D / U) {
    case 64 / U: return D == 64 ? (const void *)route_score_kernel<QD, 64 / U> : nullptr;
    case 128 / U: return D == 128 ? (const void *)route_score_kernel<QD, 128 / U> : nullptr;
    case 256 / U: return D == 256 ? (const void *)route_score_kernel<QD, 256 / U> : nullptr;
    default: return nullptr;
    }
}

}  // namespace

int launch_route(const moska_problem_t &p, const void *Q, const void *E, int32_t *ids, float *scores,
                 uint64_t *keys, hipStream_t s) {
    const int64_t rows = (int64_t)p.B * p.Hkv;
    const void *score = p.q_dtype == MOSKA_BF16 ? score_kernel_for<MOSKA_BF16>(p.D) : score_kernel_for<MOSKA_F32>(p.D);
    // a small problem is bound by launch latency: scoring and selection in one kernel, on the vector ALU
    static const int64_t lane_limit = tuning_env("MOSKA_ROUTE_LANE_LIMIT", 4 << 20);
    if (rows * p.C * p.D <= lane_limit && p.k <= 32 && p.C <= 1024) score = nullptr;
    if (score) {
        int B = p.B, Hq = p.Hq, Hkv = p.Hkv, C = p.C, k = p.k;
        int btiles = (p.B + 15) / 16, ctiles = (p.C + 15) / 16;
        int64_t want = (4096 + (int64_t)p.Hkv * btiles - 1) / ((int64_t)p.Hkv * btiles);   // ~4096 waves
        int csplit = (int)(want < 1 ? 1 : want > ctiles ? ctiles : want);
        const int64_t waves = (int64_t)p.Hkv * btiles * csplit;
        void *kargs[] = {&Q, &E, &keys, &B, &Hq, &Hkv, &C, &btiles, &csplit, &ctiles};
        if (hipLaunchKernel(score, dim3((unsigned)((waves + 3) / 4)), dim3(256), kargs, 0, s) != hipSuccess)
            return MOSKA_ERR_HIP;

        if (p.C <= 16 * kWave) {                           // keys fit in registers
            const int kpl = (p.C + kWave - 1) / kWave;
            const void *sel = kpl <= 1 ? (const void *)route_select_reg_kernel<1>
                              : kpl <= 2 ? (const void *)route_select_reg_kernel<2>
                              : kpl <= 4 ? (const void *)route_select_reg_kernel<4>
                              : kpl <= 8 ? (const void *)route_select_reg_kernel<8>
                                         : (const void *)route_select_reg_kernel<16>;
            int64_t nrows = rows;
            const uint64_t *ck = keys;
            void *sargs[] = {&ck, &ids, &scores, &nrows, &C, &k};
            if (hipLaunchKernel(sel, dim3((unsigned)((rows + 3) / 4)), dim3(4 * kWave), sargs, 0, s) != hipSuccess)
                return MOSKA_ERR_HIP;
            return hip_status(hipGetLastError());
        }
        if (p.k > 32 && p.C <= 4096) {                      // many chunks and a large k: sort the row
            const void *sel = p.C <= 2048 ? (const void *)route_sort_kernel<8> : (const void *)route_sort_kernel<16>;
            const uint64_t *ck = keys;
            void *sargs[] = {&ck, &ids, &scores, &C, &k};
            if (hipLaunchKernel(sel, dim3((unsigned)rows), dim3(256), sargs, 0, s) != hipSuccess) return MOSKA_ERR_HIP;
            return hip_status(hipGetLastError());
        }
        const size_t per_wave = (size_t)p.C * sizeof(uint64_t);
        int W = (int)((140u * 1024u) / per_wave);
        if (W < 1) return MOSKA_ERR_UNSUPPORTED;
        if (W > 4) W = 4;
        const size_t lds = per_wave * W;
        if (int rc = raise_lds_limit(route_select_kernel, lds)) return rc;
        hipLaunchKernelGGL(route_select_kernel, dim3((unsigned)((rows + W - 1) / W)), dim3(W * kWave), lds, s,
                           (const uint64_t *)keys, ids, scores, rows, C, k, W);
        return hip_status(hipGetLastError());
    }
    const size_t per_wave = (size_t)(p.D + p.C) * sizeof(double);
    int W = (int)((140u * 1024u) / per_wave);
    if (W < 1) return MOSKA_ERR_UNSUPPORTED;
    if (W > 4) W = 4;
    const size_t lds = per_wave * W;
    const unsigned grid = (unsigned)((rows + W - 1) / W);
    auto kern = p.q_dtype == MOSKA_BF16 ? route_lane_kernel<MOSKA_BF16> : route_lane_kernel<MOSKA_F32>;
    if (int rc = raise_lds_limit(kern, lds)) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(W * kWave), lds, s, Q, E, ids, scores, p.B, p.Hq, p.Hkv, p.D, p.C,
                       p.k, W);
    return hip_status(hipGetLastError());
}

}  // namespace moska
