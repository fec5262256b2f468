// Shared KV Attention and Unique KV Attention on the gfx950 matrix cores (bf16 queries, head
// size 128, bf16 or fp8-e4m3 shared store), paper Sec. III-A.
//
// Both are the same streaming problem: up to 16*NR query rows that attend to ONE key set -- the
// gathered rows of a (chunk, KV head) bucket, or the G heads of one request -- while K and V of
// that set are read from HBM exactly once.  A workgroup's NW wavefronts split the keys (32-key
// tiles, interleaved), each keeps all rows' queries and output accumulators in registers, and the
// waves' partial (max, sum, O) are combined through LDS at the end.  Nothing is staged in LDS on
// the way in: the global-memory access patterns are chosen so that what a lane loads IS its MFMA
// operand.
//
// v_mfma_f32_16x16x32_bf16 computes C[16x16] += A[16x32] * B[32x16]; lane (q = lane/16,
// x = lane%16) holds A[x][8q..8q+7], B[8q..8q+7][x] and C[4q..4q+3][x].
//
//   S^T = K Q^T      A = 16 keys x 32 dims: lane (q,x) loads 16 B of key row x   (contiguous dims)
//                    B = Q^T, resident in registers for the whole kernel
//                    C: lane (q,x) gets keys 4q..4q+3 of row x  -> a softmax row lives in the
//                       four lanes x, x+16, x+32, x+48: two cross-lane steps per statistic
//   O^T = V^T P^T    B = P^T: a lane's 8 probabilities (keys 4q..4q+3 of both 16-key blocks of a
//                       32-key tile) are used as they are -- the contraction order of the keys
//                       is free as long as V uses the same one
//                    A = V^T: lane (q,x) loads dims 8x..8x+7 of exactly those 8 keys (each load
//                       instruction covers four whole 256-byte rows) and transposes the 8x8
//                       block in registers with byte permutes; MFMA number e (0..7) then takes
//                       dim 8x+e, so a lane accumulates O[row x][32q .. 32q+31]
#include "moska_internal.h"

namespace moska {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int HD = 128;                       // head size served here
constexpr int OSTRIDE = HD + 4;               // LDS row: 128 outputs, max, sum, pad
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr uint32_t kSelLo = 0x05040100u;      // v_perm: (lo16 of b) | (lo16 of a) << 16
constexpr uint32_t kSelHi = 0x07060302u;      // v_perm: (hi16 of b) | (hi16 of a) << 16

__device__ __forceinline__ f32x4 mfma16(const uint32_t (&a)[4], const uint32_t (&b)[4], f32x4 c) {
    const u32x4 av = {a[0], a[1], a[2], a[3]}, bv = {b[0], b[1], b[2], b[3]};
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv), c,
                                                   0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // round to nearest even
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// the first head dim of the 8 that lane group q contributes to MFMA step kb of S^T = K Q^T
template <int KVD>
__device__ __forceinline__ int qk_dim0(int kb, int q) {
    if constexpr (KVD == MOSKA_BF16) return 32 * kb + 8 * q;         // 16-byte loads of bf16 keys
    else return 64 * (kb >> 1) + 16 * q + 8 * (kb & 1);              // 16-byte loads of fp8 keys
}

template <int KVD> struct TileRegs;
template <> struct TileRegs<MOSKA_BF16> {
    uint4 k[2][4];      // [16-key block][kb]
    uint4 v[8];         // [key slot]: dims 8x..8x+7
};
template <> struct TileRegs<MOSKA_FP8_E4M3> {
    uint4 k[2][2];      // [16-key block][64-dim half]: dims 64u+16q .. +15
    uint2 v[8];
};

// key of slot s (0..7) inside a 32-key tile for lane group q
__device__ __forceinline__ int slot_key(int s, int q) { return s < 4 ? 4 * q + s : 12 + 4 * q + s; }

template <int KVD>
__device__ __forceinline__ void load_tile(TileRegs<KVD> &t, const char *Kb, const char *Vb, int key0, int nkeys,
                                          int q, int x) {
    constexpr int ROWB = KVD == MOSKA_BF16 ? 2 * HD : HD;
    const int last = nkeys - 1;                      // rows past the end re-read the last row (masked later)
#pragma unroll
    for (int kblk = 0; kblk < 2; ++kblk) {
        const char *rp = Kb + (int64_t)min(key0 + 16 * kblk + x, last) * ROWB + 16 * q;
        if constexpr (KVD == MOSKA_BF16) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) t.k[kblk][kb] = *(const uint4 *)(rp + 64 * kb);
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) t.k[kblk][u] = *(const uint4 *)(rp + 64 * u);
        }
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const char *rp = Vb + (int64_t)min(key0 + slot_key(s, q), last) * ROWB;
        if constexpr (KVD == MOSKA_BF16) t.v[s] = *(const uint4 *)(rp + 16 * x);
        else t.v[s] = *(const uint2 *)(rp + 8 * x);
    }
}

template <int NR> struct WaveState {
    f32x4 o[NR][8];     // [row block][e]: O[row 16rb+x][32q + 8r + e] in component r
    float m[NR], l[NR]; // running max (log2 domain) and this lane's share of the running sum
};

// bytes (0,1) or (2,3) of w as two floats; the selector folds to a constant after unrolling
__device__ __forceinline__ f32x2 cvt2_fp8(uint32_t w, bool upper) {
    return upper ? __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true) : __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
}

// four fp8 bytes of w -> two dwords of packed bf16 (exact)
__device__ __forceinline__ void fp8x4_to_bf16x4(uint32_t w, uint32_t &d0, uint32_t &d1) {
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    d0 = __builtin_amdgcn_perm(__float_as_uint(a[1]), __float_as_uint(a[0]), kSelHi);
    d1 = __builtin_amdgcn_perm(__float_as_uint(b[1]), __float_as_uint(b[0]), kSelHi);
}

template <int NR, int KVD>
__device__ __forceinline__ void process_tile(WaveState<NR> &st, const uint32_t (&qf)[NR][4][4],
                                             const TileRegs<KVD> &t, int key0, int nkeys, float sc, int q) {
    // ---- S^T = K Q^T -----------------------------------------------------------------------
    uint32_t kf[2][4][4];
#pragma unroll
    for (int kblk = 0; kblk < 2; ++kblk) {
        if constexpr (KVD == MOSKA_BF16) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                kf[kblk][kb][0] = t.k[kblk][kb].x; kf[kblk][kb][1] = t.k[kblk][kb].y;
                kf[kblk][kb][2] = t.k[kblk][kb].z; kf[kblk][kb][3] = t.k[kblk][kb].w;
            }
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                fp8x4_to_bf16x4(t.k[kblk][u].x, kf[kblk][2 * u][0], kf[kblk][2 * u][1]);
                fp8x4_to_bf16x4(t.k[kblk][u].y, kf[kblk][2 * u][2], kf[kblk][2 * u][3]);
                fp8x4_to_bf16x4(t.k[kblk][u].z, kf[kblk][2 * u + 1][0], kf[kblk][2 * u + 1][1]);
                fp8x4_to_bf16x4(t.k[kblk][u].w, kf[kblk][2 * u + 1][2], kf[kblk][2 * u + 1][3]);
            }
        }
    }
    f32x4 s[NR][2];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb)
#pragma unroll
        for (int kblk = 0; kblk < 2; ++kblk) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) acc = mfma16(kf[kblk][kb], qf[rb][kb], acc);
            s[rb][kblk] = acc;
        }

    // ---- online softmax (log2 domain) --------------------------------------------------------
    const bool tail = key0 + 32 > nkeys;
    uint32_t pf[NR][4];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        float v[8];
#pragma unroll
        for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float z = s[rb][kblk][r] * sc;
                if (tail && key0 + 16 * kblk + 4 * q + r >= nkeys) z = -INFINITY;
                v[4 * kblk + r] = z;
            }
        float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mn = fmaxf(st.m[rb], mx);        // finite: every tile holds at least one real key
        const float alpha = __builtin_amdgcn_exp2f(st.m[rb] - mn);
        st.m[rb] = mn;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            v[i] = __builtin_amdgcn_exp2f(v[i] - mn);
            sum += v[i];
        }
        st.l[rb] = st.l[rb] * alpha + sum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int e = 0; e < 8; ++e) st.o[rb][e] *= alpha;
        }
        pf[rb][0] = pack_bf16(v[0], v[1]);
        pf[rb][1] = pack_bf16(v[2], v[3]);
        pf[rb][2] = pack_bf16(v[4], v[5]);
        pf[rb][3] = pack_bf16(v[6], v[7]);
    }

    // ---- O^T += V^T P^T ----------------------------------------------------------------------
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        uint32_t vf[4];
        if constexpr (KVD == MOSKA_BF16) {
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                const uint4 a = t.v[2 * pr + 1], b = t.v[2 * pr];
                const uint32_t wa = (e >> 1) == 0 ? a.x : (e >> 1) == 1 ? a.y : (e >> 1) == 2 ? a.z : a.w;
                const uint32_t wb = (e >> 1) == 0 ? b.x : (e >> 1) == 1 ? b.y : (e >> 1) == 2 ? b.z : b.w;
                vf[pr] = __builtin_amdgcn_perm(wa, wb, (e & 1) ? kSelHi : kSelLo);
            }
        } else {
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                const uint32_t wa = e < 4 ? t.v[2 * pr + 1].x : t.v[2 * pr + 1].y;
                const uint32_t wb = e < 4 ? t.v[2 * pr].x : t.v[2 * pr].y;
                const f32x2 fa = cvt2_fp8(wa, (e & 2) != 0), fb = cvt2_fp8(wb, (e & 2) != 0);
                vf[pr] = __builtin_amdgcn_perm(__float_as_uint(fa[e & 1]), __float_as_uint(fb[e & 1]), kSelHi);
            }
        }
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) st.o[rb][e] = mfma16(vf, pf[rb], st.o[rb][e]);
    }
}

// Stream keys [0,nkeys) of one key set; wave `wave` of NW takes tiles wave, wave+NW, ...
template <int NR, int KVD, int NW>
__device__ __forceinline__ void attend(WaveState<NR> &st, const uint32_t (&qf)[NR][4][4], const char *Kb,
                                       const char *Vb, int nkeys, float sc, int wave, int q, int x) {
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        st.m[rb] = -INFINITY;
        st.l[rb] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[rb][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int nt = (nkeys + 31) >> 5;
    TileRegs<KVD> ta, tb;                          // two tiles in flight: the next one loads while this one computes
    int t = wave;
    if (t < nt) load_tile<KVD>(ta, Kb, Vb, 32 * t, nkeys, q, x);
    while (t < nt) {
        const int t2 = t + NW;
        if (t2 < nt) load_tile<KVD>(tb, Kb, Vb, 32 * t2, nkeys, q, x);
        process_tile<NR, KVD>(st, qf, ta, 32 * t, nkeys, sc, q);
        if (t2 >= nt) break;
        const int t3 = t2 + NW;
        if (t3 < nt) load_tile<KVD>(ta, Kb, Vb, 32 * t3, nkeys, q, x);
        process_tile<NR, KVD>(st, qf, tb, 32 * t2, nkeys, sc, q);
        t = t3;
    }
}

// Merge the NW waves' states pairwise through LDS and let wave 0 write the rows.
// orow[rb]: index of row 16rb+x in part_LSE (part_O row = orow*HD), or -1 for a padding row.
template <int NR, int NW>
__device__ __forceinline__ void combine_and_store(WaveState<NR> &st, float *lds, int wave, int q, int x,
                                                  const int64_t (&orow)[NR], float vmul, float *part_O,
                                                  float *part_LSE) {
    constexpr int R = 16 * NR;
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        float l = st.l[rb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        st.l[rb] = l;
    }
#pragma unroll
    for (int s = NW / 2; s >= 1; s >>= 1) {
        if (wave >= s && wave < 2 * s) {
            float *buf = lds + (size_t)(wave - s) * R * OSTRIDE;
#pragma unroll
            for (int rb = 0; rb < NR; ++rb) {
                float *row = buf + (16 * rb + x) * OSTRIDE;
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int r = 0; r < 4; ++r) row[32 * q + 8 * r + e] = st.o[rb][e][r];
                if (q == 0) {
                    row[HD] = st.m[rb];
                    row[HD + 1] = st.l[rb];
                }
            }
        }
        __syncthreads();
        if (wave < s) {
            const float *buf = lds + (size_t)wave * R * OSTRIDE;
#pragma unroll
            for (int rb = 0; rb < NR; ++rb) {
                const float *row = buf + (16 * rb + x) * OSTRIDE;
                const float m2 = row[HD], l2 = row[HD + 1];
                const float mn = fmaxf(st.m[rb], m2);
                const float a1 = st.m[rb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(st.m[rb] - mn);
                const float a2 = m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int r = 0; r < 4; ++r) st.o[rb][e][r] = st.o[rb][e][r] * a1 + row[32 * q + 8 * r + e] * a2;
                st.l[rb] = st.l[rb] * a1 + l2 * a2;
                st.m[rb] = mn;
            }
        }
        __syncthreads();
    }
    if (wave == 0) {
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) {
            if (orow[rb] < 0) continue;
            const float l = st.l[rb];
            const float inv = l > 0.f ? vmul / l : 0.f;
            float *o = part_O + orow[rb] * HD + 32 * q;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float4 lo = {st.o[rb][0][r] * inv, st.o[rb][1][r] * inv, st.o[rb][2][r] * inv, st.o[rb][3][r] * inv};
                const float4 hi = {st.o[rb][4][r] * inv, st.o[rb][5][r] * inv, st.o[rb][6][r] * inv, st.o[rb][7][r] * inv};
                *(float4 *)(o + 8 * r) = lo;
                *(float4 *)(o + 8 * r + 4) = hi;
            }
            if (q == 0) part_LSE[orow[rb]] = l > 0.f ? (st.m[rb] + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
        }
    }
}

// Q^T operand of row (element offset qoff into Q, or zeros for a padding row)
template <int KVD>
__device__ __forceinline__ void load_q(uint32_t (&qf)[4][4], const void *Q, int64_t qoff, bool valid, int q) {
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        uint4 v = {0u, 0u, 0u, 0u};
        if (valid) v = *(const uint4 *)((const uint16_t *)Q + qoff + qk_dim0<KVD>(kb, q));
        qf[kb][0] = v.x; qf[kb][1] = v.y; qf[kb][2] = v.z; qf[kb][3] = v.w;
    }
}

template <int NR, int KVD, int NW>
__global__ __launch_bounds__(NW * 64) void shared_mfma_kernel(SharedArgs a, int Hq, int Hkv, int C, int L, int k,
                                                               float scale) {
    __shared__ float comb[(NW / 2) * 16 * NR * OSTRIDE];
    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous range of the
    // tile list so the tiles of one bucket (which re-read the same chunk) share an L2.
    const int ntiles = a.tile_hdr[0];
    const int per = (ntiles + 7) >> 3, slot = blockIdx.x >> 3;
    const int w = (blockIdx.x & 7) * per + slot;
    if (slot >= per || w >= ntiles) return;
    const int bkt = a.tiles[2 * w], row0 = a.tiles[2 * w + 1];
    const int h = bkt / C, c = bkt - h * C, G = Hq / Hkv;
    const int beg = a.off[bkt], rows = (a.off[bkt + 1] - beg) * G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, q = lane >> 4, x = lane & 15;

    uint32_t qf[NR][4][4];
    int64_t orow[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int rr = row0 + 16 * rb + x;
        const bool valid = rr < rows;
        int64_t qoff = 0;
        orow[rb] = -1;
        if (valid) {
            const int item = a.items[beg + rr / G], g = rr % G;
            const int b = item / k, j = item - b * k;
            const int64_t bh = (int64_t)b * Hq + h * G + g;
            qoff = bh * HD;
            orow[rb] = bh * (k + 1) + j;
        }
        load_q<KVD>(qf[rb], a.Q, qoff, valid, q);
    }
    const float kmul = a.scale_k ? a.scale_k[c * Hkv + h] : 1.f;
    const float vmul = a.scale_v ? a.scale_v[c * Hkv + h] : 1.f;
    constexpr int ESZ = KVD == MOSKA_BF16 ? 2 : 1;
    const int64_t base = ((int64_t)c * Hkv + h) * L * HD * ESZ;
    WaveState<NR> st;
    attend<NR, KVD, NW>(st, qf, (const char *)a.Ks + base, (const char *)a.Vs + base, L, scale * kmul * kLog2e, wave,
                        q, x);
    combine_and_store<NR, NW>(st, comb, wave, q, x, orow, vmul, a.part_O, a.part_LSE);
}

template <int NR, int NW>
__global__ __launch_bounds__(NW * 64) void unique_mfma_kernel(UniqueArgs a, int Hq, int Hkv, int U, int k,
                                                               float scale) {
    __shared__ float comb[(NW / 2) * 16 * NR * OSTRIDE];
    const int G = Hq / Hkv, gt = (G + 16 * NR - 1) / (16 * NR);
    const int bh = blockIdx.x / gt, g0 = (blockIdx.x % gt) * 16 * NR;
    const int b = bh / Hkv, h = bh - b * Hkv;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, q = lane >> 4, x = lane & 15;
    uint32_t qf[NR][4][4];
    int64_t orow[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int g = g0 + 16 * rb + x;
        const bool valid = g < G;
        const int64_t row = (int64_t)b * Hq + h * G + (valid ? g : 0);
        orow[rb] = valid ? row * (k + 1) + k : -1;
        load_q<MOSKA_BF16>(qf[rb], a.Q, row * HD, valid, q);
    }
    const int nkeys = a.unique_len ? min(max(a.unique_len[b], 0), U) : U;
    const int64_t base = ((int64_t)b * Hkv + h) * U * HD * 2;
    WaveState<NR> st;
    attend<NR, MOSKA_BF16, NW>(st, qf, (const char *)a.Ku + base, (const char *)a.Vu + base, nkeys, scale * kLog2e,
                               wave, q, x);
    combine_and_store<NR, NW>(st, comb, wave, q, x, orow, 1.f, a.part_O, a.part_LSE);
}

}  // namespace

int launch_shared_mfma(const moska_problem_t &p, const SharedArgs &a, int MT, hipStream_t s) {
    constexpr int NW = 4;
    const int64_t tmax = max_tiles(p, MT);
    if (tmax == 0) return MOSKA_OK;
    const unsigned grid = (unsigned)(((tmax + 7) / 8) * 8);
    const bool fp8 = p.shared_kv_dtype == MOSKA_FP8_E4M3;
#define MOSKA_LAUNCH_SHARED(NR)                                                                                   \
    do {                                                                                                           \
        if (fp8)                                                                                                   \
            hipLaunchKernelGGL((shared_mfma_kernel<NR, MOSKA_FP8_E4M3, NW>), dim3(grid), dim3(NW * 64), 0, s, a,   \
                               p.Hq, p.Hkv, p.C, p.L, p.k, p.scale);                                               \
        else                                                                                                       \
            hipLaunchKernelGGL((shared_mfma_kernel<NR, MOSKA_BF16, NW>), dim3(grid), dim3(NW * 64), 0, s, a, p.Hq, \
                               p.Hkv, p.C, p.L, p.k, p.scale);                                                     \
    } while (0)
    if (MT == 16) MOSKA_LAUNCH_SHARED(1);
    else if (MT == 32) MOSKA_LAUNCH_SHARED(2);
    else if (MT == 64) MOSKA_LAUNCH_SHARED(4);
    else return MOSKA_ERR_UNSUPPORTED;
#undef MOSKA_LAUNCH_SHARED
    return hip_status(hipGetLastError());
}

int launch_unique_mfma(const moska_problem_t &p, const UniqueArgs &a, hipStream_t s) {
    constexpr int NW = 4;
    const int G = p.Hq / p.Hkv;
    const int NR = G <= 16 ? 1 : G <= 32 ? 2 : 4;
    const int gt = (G + 16 * NR - 1) / (16 * NR);
    const unsigned grid = (unsigned)((int64_t)p.B * p.Hkv * gt);
    if (NR == 1)
        hipLaunchKernelGGL((unique_mfma_kernel<1, NW>), dim3(grid), dim3(NW * 64), 0, s, a, p.Hq, p.Hkv, p.U_max, p.k,
                           p.scale);
    else if (NR == 2)
        hipLaunchKernelGGL((unique_mfma_kernel<2, NW>), dim3(grid), dim3(NW * 64), 0, s, a, p.Hq, p.Hkv, p.U_max, p.k,
                           p.scale);
    else
        hipLaunchKernelGGL((unique_mfma_kernel<4, NW>), dim3(grid), dim3(NW * 64), 0, s, a, p.Hq, p.Hkv, p.U_max, p.k,
                           p.scale);
    return hip_status(hipGetLastError());
}

}  // namespace moska
