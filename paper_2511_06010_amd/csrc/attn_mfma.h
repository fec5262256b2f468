// Device code of the MFMA streaming attention (Shared KV Attention and Unique KV Attention,
// paper Sec. III-A) for bf16 queries, head size 128 and a bf16 or fp8-e4m3 key/value store.
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
#pragma once

#include "moska_internal.h"

namespace moska {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int HD = 128;                       // head size served here
constexpr int OSTRIDE = HD + 4;               // LDS row: 128 outputs, max, sum, pad
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazy = 8.f;                  // log2 units, see softmax_tile
constexpr uint32_t kSelLo = 0x05040100u;      // v_perm: (lo16 of b) | (lo16 of a) << 16
constexpr uint32_t kSelHi = 0x07060302u;      // v_perm: (hi16 of b) | (hi16 of a) << 16

__device__ __forceinline__ f32x4 mfma16(const uint32_t (&a)[4], const uint32_t (&b)[4], f32x4 c) {
    const u32x4 av = {a[0], a[1], a[2], a[3]}, bv = {b[0], b[1], b[2], b[3]};
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv), c,
                                                   0, 0, 0);
}

// acc + lo + hi of a packed pair of bf16
__device__ __forceinline__ float dot2_ones(uint32_t pair, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc,
                                           false);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // round to nearest even
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}


// Reductions over the four lanes x, x+16, x+32, x+48 that share a query row, on the vector ALU
// (v_permlane16_swap / v_permlane32_swap hand every lane both members of its xor-16 / xor-32 pair).
__device__ __forceinline__ float row_lanes_max(float v) {
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float row_lanes_sum(float v) {
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <int KVD> constexpr int row_bytes() { return KVD == MOSKA_BF16 ? 2 * HD : HD; }

// the first head dim of the 8 that lane group q contributes to MFMA step kb of S^T = K Q^T
template <int KVD>
__device__ __forceinline__ int qk_dim0(int kb, int q) {
    if constexpr (KVD == MOSKA_BF16) return 32 * kb + 8 * q;         // 16-byte loads of bf16 keys
    else return 64 * (kb >> 1) + 16 * q + 8 * (kb & 1);              // 16-byte loads of fp8 keys
}

template <int KVD> struct TileK;
template <> struct TileK<MOSKA_BF16> { uint4 k[2][4]; };       // [16-key block][kb]
template <> struct TileK<MOSKA_FP8_E4M3> { uint4 k[2][2]; };   // [16-key block][64-dim half]
template <int KVD> struct TileV;
template <> struct TileV<MOSKA_BF16> { uint4 v[8]; };          // [key slot]: dims 8x..8x+7
template <> struct TileV<MOSKA_FP8_E4M3> { uint2 v[8]; };

// row (inside a 32-key tile) of key slot s (0..7) for lane group q
__device__ __forceinline__ constexpr int slot_row(int s) { return s < 4 ? s : 12 + s; }   // + 4q

// K and V of a key set are read through raw buffer resources that span exactly the set's
// nkeys rows: the hardware range check returns zeros for rows past the end, so ragged tails need
// no clamping (their scores are masked in the softmax).  A load's address is
// voffset (tile start + the lane's fixed offset) + a compile-time constant.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t key_set_rsrc(const char *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)bytes, 0x00020000);
}

// A lane's byte offsets inside a tile; tile t of a key set starts at byte 32*t*ROWB.
template <int KVD> struct LaneOff {
    uint32_t k, v;
    __device__ __forceinline__ LaneOff(int q, int x)
        : k((uint32_t)(x * row_bytes<KVD>() + 16 * q)),
          v((uint32_t)(4 * q * row_bytes<KVD>() + (KVD == MOSKA_BF16 ? 16 : 8) * x)) {}
};

__device__ __forceinline__ uint4 as_uint4(u32x4 v) { return uint4{v[0], v[1], v[2], v[3]}; }

// AUX is the cache-policy field of the buffer load: 0 = default, 2 = non-temporal (streamed once;
// measured ~12% more HBM read bandwidth than the default policy on this part).
template <int KVD, int AUX>
__device__ __forceinline__ void load_k(TileK<KVD> &t, __amdgpu_buffer_rsrc_t rk, const LaneOff<KVD> &lo, int tile) {
    constexpr int ROWB = row_bytes<KVD>();
    constexpr int NLD = KVD == MOSKA_BF16 ? 4 : 2;
    const uint32_t off = (uint32_t)tile * (32u * ROWB) + lo.k;
#pragma unroll
    for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            t.k[kblk][i] = as_uint4(__builtin_amdgcn_raw_buffer_load_b128(rk, off + kblk * 16 * ROWB + 64 * i, 0, AUX));
}

template <int KVD, int AUX>
__device__ __forceinline__ void load_v(TileV<KVD> &t, __amdgpu_buffer_rsrc_t rv, const LaneOff<KVD> &lo, int tile) {
    constexpr int ROWB = row_bytes<KVD>();
    const uint32_t off = (uint32_t)tile * (32u * ROWB) + lo.v;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if constexpr (KVD == MOSKA_BF16) {
            t.v[s] = as_uint4(__builtin_amdgcn_raw_buffer_load_b128(rv, off + slot_row(s) * ROWB, 0, AUX));
        } else {
            const auto w = __builtin_amdgcn_raw_buffer_load_b64(rv, off + slot_row(s) * ROWB, 0, AUX);
            t.v[s] = uint2{w[0], w[1]};
        }
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
    // v_cvt_scalef32_pk_bf16_fp8: two bytes -> two bf16 per instruction (scale 1)
    d0 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false));
    d1 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true));
}

__device__ __forceinline__ uint32_t word(const uint4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// S^T = K Q^T for one 32-key tile: s[rb][kblk] component r = key 16*kblk + 4q + r, row 16*rb + x
template <int NR, int KVD>
__device__ __forceinline__ void qk_tile(f32x4 (&s)[NR][2], const uint32_t (&qf)[NR][4][4], const TileK<KVD> &t) {
#pragma unroll
    for (int kblk = 0; kblk < 2; ++kblk) {
        uint32_t kf[4][4];
        if constexpr (KVD == MOSKA_BF16) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int i = 0; i < 4; ++i) kf[kb][i] = word(t.k[kblk][kb], i);
        } else {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                fp8x4_to_bf16x4(t.k[kblk][u].x, kf[2 * u][0], kf[2 * u][1]);
                fp8x4_to_bf16x4(t.k[kblk][u].y, kf[2 * u][2], kf[2 * u][3]);
                fp8x4_to_bf16x4(t.k[kblk][u].z, kf[2 * u + 1][0], kf[2 * u + 1][1]);
                fp8x4_to_bf16x4(t.k[kblk][u].w, kf[2 * u + 1][2], kf[2 * u + 1][3]);
            }
        }
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) acc = mfma16(kf[kb], qf[rb][kb], acc);
            s[rb][kblk] = acc;
        }
    }
}

// Number of keys row block rb may see: one count for all rows, or one per row block (each lane its
// own row's), for query tokens at different positions of the same context.
__device__ __forceinline__ int limit_of(int nkeys, int) { return nkeys; }
template <int NR> __device__ __forceinline__ int limit_of(const int (&lim)[NR], int rb) { return lim[rb]; }

// online softmax in the log2 domain; produces the P^T operands and rescales O when a max moved.
// sc > 0 folds the logit scale, the dequantisation factor of the keys and log2(e).
// TAIL: keys at or past the row's limit are masked (a row may then have no key at all yet: its
// reference stays -inf and its probabilities are zero).
// NA: the wave's first NA row blocks are worked on, the others left alone (NR <= 2 only).
template <int NR, bool TAIL, int NA = NR, typename LIM>
__device__ __forceinline__ void softmax_tile(WaveState<NR> &st, const f32x4 (&s)[NR][2], uint32_t (&pf)[NR][4],
                                             int key0, const LIM &nkeys, float sc, int q) {
    static_assert(NA == NR || NR <= 2, "a wave with four row blocks works on all of them");
    // with one count for all rows every masked tile still holds a key of every row; with per-row
    // counts a row may have none so far (m = -inf) and must come out of the tile unchanged
    constexpr bool EMPTY_ROWS = TAIL && !__is_same(LIM, int);
    // The reference point of a row moves only when the tile's maximum exceeds it by more than kLazy
    // (a factor 2^kLazy in the probabilities, harmless in fp32 sums and in bf16's exponent range);
    // otherwise nothing is rescaled.  First tile: m = -inf, always moves.
    if constexpr (NR <= 2) {
        // Every lane tests its own eight scores against the row's threshold; only if some lane of
        // the wave is over it are the row maxima completed across lanes and the references moved: ONE
        // wave-uniform branch, no cross-lane work on the usual path.
        float v[NR][8], mx[NR];
        bool over = false;
#pragma unroll
        for (int rb = 0; rb < NA; ++rb) {
#pragma unroll
            for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float z = s[rb][kblk][r];
                    if (TAIL && key0 + 16 * kblk + 4 * q + r >= limit_of(nkeys, rb)) z = -INFINITY;   // rows past the end read as 0
                    v[rb][4 * kblk + r] = z;
                }
            const float *w = v[rb];
            mx[rb] = fmaxf(fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3])), fmaxf(fmaxf(w[4], w[5]), fmaxf(w[6], w[7])));
            over |= mx[rb] * sc > st.m[rb] + kLazy;
        }
        const bool resc = __any(over);
        float alpha[NR];
#pragma unroll
        for (int rb = 0; rb < NA; ++rb) alpha[rb] = 1.f;
        if (resc) {
#pragma unroll
            for (int rb = 0; rb < NA; ++rb) {
                const float rmx = row_lanes_max(mx[rb]) * sc;
                const bool moved = rmx > st.m[rb] + kLazy;
                const float mn = moved ? rmx : st.m[rb];
                alpha[rb] = __builtin_amdgcn_exp2f(st.m[rb] - mn);            // exactly 1 for rows that stay
                if (EMPTY_ROWS && !moved) alpha[rb] = 1.f;                    // (-inf) - (-inf)
                st.m[rb] = mn;
                st.l[rb] *= alpha[rb];
            }
        }
        if (resc) {
#pragma unroll
            for (int rb = 0; rb < NA; ++rb)
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int r = 0; r < 4; ++r) st.o[rb][e][r] *= alpha[rb];
        }
#pragma unroll
        for (int rb = 0; rb < NA; ++rb) {
            const float mn = EMPTY_ROWS && st.m[rb] == -INFINITY ? 0.f : st.m[rb];   // no key yet: exp2(-inf) = 0 below
#pragma unroll
            for (int i = 0; i < 8; ++i) v[rb][i] = __builtin_amdgcn_exp2f(fmaf(v[rb][i], sc, -mn));
            pf[rb][0] = pack_bf16(v[rb][0], v[rb][1]);
            pf[rb][1] = pack_bf16(v[rb][2], v[rb][3]);
            pf[rb][2] = pack_bf16(v[rb][4], v[rb][5]);
            pf[rb][3] = pack_bf16(v[rb][6], v[rb][7]);
            // the row sum takes the probabilities as the P V product sees them (rounded to bf16), two per
            // instruction: v_dot2c_f32_bf16 against a pair of ones
#pragma unroll
            for (int i = 0; i < 4; ++i) st.l[rb] = dot2_ones(pf[rb][i], st.l[rb]);
        }
    } else {
        // four row blocks: one at a time, to keep the live scores within the register file
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) {
            float v[8];
#pragma unroll
            for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float z = s[rb][kblk][r];
                    if (TAIL && key0 + 16 * kblk + 4 * q + r >= limit_of(nkeys, rb)) z = -INFINITY;   // rows past the end read as 0
                    v[4 * kblk + r] = z;
                }
            float mx = fmaxf(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])), fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7])));
            mx = row_lanes_max(mx) * sc;
            const bool moved = mx > st.m[rb] + kLazy;                  // first tile with a key: m = -inf, moves
            const float mn = moved ? mx : st.m[rb];
            float alpha = __builtin_amdgcn_exp2f(st.m[rb] - mn);       // exactly 1 unless the reference moved
            if (EMPTY_ROWS && !moved) alpha = 1.f;                     // (-inf) - (-inf)
            st.m[rb] = mn;
            const float off = EMPTY_ROWS && mn == -INFINITY ? 0.f : mn;   // no key yet: exp2(-inf) = 0 below
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[i] = __builtin_amdgcn_exp2f(fmaf(v[i], sc, -off));
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
    }
}

// O^T += V^T P^T for one 32-key tile
template <int NR, int KVD>
__device__ __forceinline__ void pv_tile(WaveState<NR> &st, const TileV<KVD> &t, const uint32_t (&pf)[NR][4]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        uint32_t vf[4];
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            if constexpr (KVD == MOSKA_BF16) {
                vf[pr] = __builtin_amdgcn_perm(word(t.v[2 * pr + 1], e >> 1), word(t.v[2 * pr], e >> 1),
                                               (e & 1) ? kSelHi : kSelLo);
            } else {
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
// A tile's registers are refilled with a later tile of the wave as soon as the MFMAs that read
// them have issued (loads past the end of the set are dropped by the range check, so refills need
// no branch).  NKB = 1: one key tile and one value tile in flight per wave, latency hidden by the
// other waves of the SIMD.  NKB = 2: two key tiles in flight, for the 64-row kernels whose
// register footprint allows only one wave per SIMD.
// lim: how many of the keys each row may see -- nkeys itself (an int), or per row block the lane's
// own row's count (<= nkeys); nsafe <= every row's count: tiles below it need no masking.
template <int NR, int KVD, int NW, int AUX, int NKB, typename LIM>
__device__ __forceinline__ void attend(WaveState<NR> &st, const uint32_t (&qf)[NR][4][4], const char *Kb,
                                       const char *Vb, int nkeys, int nsafe, const LIM &lim, float sc, int wave,
                                       int q, int x) {
    static_assert(NKB == 1 || NKB == 2, "key tiles in flight");
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        st.m[rb] = -INFINITY;
        st.l[rb] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[rb][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int nfull = nsafe >> 5;                  // tiles that every row sees whole
    const LaneOff<KVD> lo(q, x);
    const __amdgpu_buffer_rsrc_t rk = key_set_rsrc(Kb, (uint32_t)nkeys * row_bytes<KVD>());
    const __amdgpu_buffer_rsrc_t rv = key_set_rsrc(Vb, (uint32_t)nkeys * row_bytes<KVD>());
    TileK<KVD> tk[NKB];
    TileV<KVD> tv;
    f32x4 s[NR][2];
    uint32_t pf[NR][4];
    // one tile: scores, refill the key registers NKB tiles ahead, softmax, output, refill values
    auto step = [&](TileK<KVD> &k, int tt) {
        qk_tile<NR, KVD>(s, qf, k);
        load_k<KVD, AUX>(k, rk, lo, tt + NKB * NW);
        softmax_tile<NR, false>(st, s, pf, 32 * tt, nkeys, sc, q);
        pv_tile<NR, KVD>(st, tv, pf);
        load_v<KVD, AUX>(tv, rv, lo, tt + NW);
    };
    int t = wave;
    if (t < nfull) {
        load_k<KVD, AUX>(tk[0], rk, lo, t);
        load_v<KVD, AUX>(tv, rv, lo, t);
        if constexpr (NKB == 2) {
            load_k<KVD, AUX>(tk[1], rk, lo, t + NW);
            while (t + NW < nfull) {
                step(tk[0], t);
                step(tk[1], t + NW);
                t += 2 * NW;
            }
            if (t < nfull) step(tk[0], t);
        } else {
            do {
                step(tk[0], t);
                t += NW;
            } while (t < nfull);
        }
    }
    // the remaining tiles (one ragged tile; a few when the rows' counts differ) are masked per row
    const int ntiles = (nkeys + 31) >> 5;
    for (int tt = nfull + ((wave - nfull % NW + NW) % NW); tt < ntiles; tt += NW) {
        load_k<KVD, AUX>(tk[0], rk, lo, tt);
        load_v<KVD, AUX>(tv, rv, lo, tt);
        qk_tile<NR, KVD>(s, qf, tk[0]);
        softmax_tile<NR, true>(st, s, pf, 32 * tt, lim, sc, q);
        pv_tile<NR, KVD>(st, tv, pf);
    }
}

// Partial rows are written in pieces of at least 64 contiguous bytes with the non-temporal hint.
// Mixed into a saturated K/V read stream, plain write-back stores of these rows cost far more than
// their bytes (measured at 256 requests x 8 chunks: 34 MB of partials stretch a 0.61 ms stream to
// 0.71 ms, to 0.65 ms with the hint).  The 4-byte LSE values stay write-back, so that the L2 can
// assemble lines.
// NT = false for the slices of a split run: the combine kernel reads them back at once, so they stay
// write-back.  (A compile-time choice: the compiler folds a run-time choice between two otherwise
// identical stores into one plain store.)
template <bool NT> __device__ __forceinline__ void store_partial16(float *p, const f32x4 &v) {
    if constexpr (NT) __builtin_nontemporal_store(v, (f32x4 *)p);
    else *(f32x4 *)p = v;
}

// Normalise and write the rows a wave of the LDS-staged kernels holds (st.l already summed over the
// row's four lanes): component r of o[rb][e] is dim 16e + 4q + r (operands from the LDS transpose
// read).  orow[rb]: index of row 16rb+x in part_LSE (part_O row = orow*HD), or -1 for a padding row.
template <int NR, bool NT>
__device__ __forceinline__ void store_rows(const WaveState<NR> &st, int q, const int64_t (&orow)[NR], float vmul,
                                           float *part_O, float *part_LSE) {
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        if (orow[rb] < 0) continue;
        const float l = st.l[rb];
        const float inv = l > 0.f ? vmul / l : 0.f;
        float *o = part_O + orow[rb] * HD + 4 * q;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const f32x4 v = {st.o[rb][e][0] * inv, st.o[rb][e][1] * inv, st.o[rb][e][2] * inv, st.o[rb][e][3] * inv};
            store_partial16<NT>(o + 16 * e, v);
        }
        if (q == 0) part_LSE[orow[rb]] = l > 0.f ? (st.m[rb] + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
    }
}

// Merge the NW waves' states pairwise through LDS and write the rows (all NW*64 threads that share
// `lds` must call this, tid = 0 .. NW*64-1: it contains workgroup barriers).
template <int NR, int NW, bool NT>
__device__ __forceinline__ void combine_and_store(WaveState<NR> &st, float *lds, int tid, int wave, int q, int x,
                                                  const int64_t (&orow)[NR], float vmul, float *part_O,
                                                  float *part_LSE) {
    constexpr int R = 16 * NR;
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        st.l[rb] = row_lanes_sum(st.l[rb]);
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
    // Wave 0 holds the result.  Its normalised rows go through LDS once more so that they leave as
    // whole 512-byte rows (two per store instruction, all waves storing) with the non-temporal hint.
    if (wave == 0) {
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) {
            float *row = lds + (16 * rb + x) * OSTRIDE;
            const float l = st.l[rb];
            const float inv = l > 0.f ? vmul / l : 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int r = 0; r < 4; ++r) row[32 * q + 8 * r + e] = st.o[rb][e][r] * inv;
            if (q == 0) {
                *(int64_t *)(row + HD + 2) = orow[rb];
                if (orow[rb] >= 0)
                    part_LSE[orow[rb]] = l > 0.f ? (st.m[rb] + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
            }
        }
    }
    __syncthreads();
    const int col = tid & 31;
    for (int rr = tid >> 5; rr < R; rr += 2 * NW) {
        const float *row = lds + rr * OSTRIDE;
        const int64_t o = *(const int64_t *)(row + HD + 2);
        if (o >= 0) store_partial16<NT>(part_O + o * HD + 4 * col, *(const f32x4 *)(row + 4 * col));
    }
}

// Q^T operand of a row (element offset qoff into Q, or zeros for a padding row)
template <int KVD>
__device__ __forceinline__ void load_q(uint32_t (&qf)[4][4], const void *Q, int64_t qoff, bool valid, int q) {
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        uint4 v = {0u, 0u, 0u, 0u};
        if (valid) v = *(const uint4 *)((const uint16_t *)Q + qoff + qk_dim0<KVD>(kb, q));
        qf[kb][0] = v.x; qf[kb][1] = v.y; qf[kb][2] = v.z; qf[kb][3] = v.w;
    }
}

// Slice sp of nsplit of a chunk's L keys, in whole multiples of `gran` keys: first key and count.
__device__ __forceinline__ void key_slice(int L, int nsplit, int sp, int gran, int &k0, int &nk) {
    const int per = ((L + nsplit - 1) / nsplit + gran - 1) / gran * gran;
    k0 = min(sp * per, L);
    nk = min(per, L - k0);
}

// Where a shared-attention row goes: slot j of row bh, or slice sp of that slot in the split
// workspace (combined afterwards by shared_split_combine_kernel).
__device__ __forceinline__ int64_t shared_out_row(const SharedArgs &a, int64_t bh, int j, int k, int sp) {
    return a.nsplit > 1 ? (bh * k + j) * a.nsplit + sp : bh * (k + 1) + j;
}

// Tile (bkt, row0) of Shared KV Attention on the streaming path: up to 16*NR gathered rows of
// bucket bkt against (slice blockIdx.y of) its chunk, by the NW*64 threads tid = 0 .. NW*64-1.
// comb: their LDS for the cross-wave merge, (NW/2)*16*NR*OSTRIDE floats.
template <int NR, int KVD, int NW, int AUX, int NKB, bool SPLIT>
__device__ __forceinline__ void stream_tile(const SharedArgs &a, int bkt, int row0, int Hq, int Hkv, int C, int L,
                                            int k, float scale, float *comb, int tid) {
    const int h = bkt / C, c = bkt - h * C, G = Hq / Hkv;
    const int beg = a.off[bkt], rows = (a.off[bkt + 1] - beg) * G;
    const int lane = tid & 63, q = lane >> 4, x = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps tile indices in SGPRs

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
            orow[rb] = shared_out_row(a, bh, j, k, blockIdx.y);
        }
        load_q<KVD>(qf[rb], a.Q, qoff, valid, q);
    }
    const float kmul = a.scale_k ? a.scale_k[c * Hkv + h] : 1.f;
    const float vmul = a.scale_v ? a.scale_v[c * Hkv + h] : 1.f;
    int k0, nk;
    key_slice(L, a.nsplit, blockIdx.y, 32, k0, nk);
    const int64_t base = (((int64_t)c * Hkv + h) * L + k0) * row_bytes<KVD>();
    WaveState<NR> st;
    attend<NR, KVD, NW, AUX, NKB>(st, qf, (const char *)a.Ks + base, (const char *)a.Vs + base, nk, nk, nk,
                                  scale * kmul * kLog2e, wave, q, x);
    combine_and_store<NR, NW, !SPLIT>(st, comb, tid, wave, q, x, orow, vmul, SPLIT ? a.split_O : a.part_O,
                                      SPLIT ? a.split_LSE : a.part_LSE);
}

// Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous range of the work
// list so the tiles of one bucket (which re-read the same chunk) share an L2.  bx: the workgroup's
// number inside a range of workgroups that starts at a multiple of 8.  Returns the work item
// inside [0, n) or -1 if this workgroup has none.
__device__ __forceinline__ int xcd_tile_index(int bx, int n) {
    const int per = (n + 7) >> 3, slot = bx >> 3;
    const int w = (bx & 7) * per + slot;
    return (slot >= per || w >= n) ? -1 : w;
}

// Up to 32 rows fit in 256 registers per lane: asking for two waves per SIMD keeps the MFMA
// accumulators in architectural VGPRs, where the softmax rescale can touch them without copies.
constexpr int min_waves(int NR) { return NR == 1 ? 3 : NR == 2 ? 2 : 1; }

// Unique KV Attention: a workgroup serves (up to 16*NR of) the T*G query rows of one (request, KV
// head) pair -- row t*G + g is query token t, head g of the group -- over one of nsplit contiguous
// slices of the request's context (nsplit = 1: all of it, the result goes straight to slot k;
// otherwise to the split workspace, combined afterwards).  Token t sees the first len - (T-1-t) keys.
template <int NR, int NW, int AUX, int NKB, bool SPLIT>
__global__ __launch_bounds__(NW * 64, min_waves(NR)) void unique_mfma_kernel(UniqueArgs a, int Hq, int Hkv, int U, int k,
                                                                              float scale, int T) {
    __shared__ float comb[(NW / 2) * 16 * NR * OSTRIDE];
    const int G = Hq / Hkv, R = T * G, gt = (R + 16 * NR - 1) / (16 * NR), ns = a.nsplit;
    const int sp = blockIdx.x % ns, wg = blockIdx.x / ns;
    const int bh = wg / gt, r0 = (wg % gt) * 16 * NR;
    const int b = bh / Hkv, h = bh - b * Hkv;
    const int lane = threadIdx.x & 63, q = lane >> 4, x = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keeps tile indices in SGPRs
    const int len = a.unique_len ? min(max(a.unique_len[b], 0), U) : U;
    const int per = ((len + ns - 1) / ns + 31) & ~31;       // keys per slice, whole 32-key tiles
    const int k0 = min(sp * per, len), nkeys = min(per, len - k0);
    uint32_t qf[NR][4][4];
    int64_t orow[NR];
    int lim[NR];                                            // keys of this slice the lane's rows may see
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int r = r0 + 16 * rb + x;
        const bool valid = r < R;
        const int t = valid ? r / G : T - 1, g = valid ? r - t * G : 0;
        const int64_t row = ((int64_t)b * T + t) * Hq + h * G + g;
        orow[rb] = !valid ? -1 : ns > 1 ? row * ns + sp : row * (k + 1) + k;
        lim[rb] = min(max(len - (T - 1 - t) - k0, 0), nkeys);
        load_q<MOSKA_BF16>(qf[rb], a.Q, row * HD, valid, q);
    }
    // the workgroup's earliest token bounds what every row sees
    const int t_first = min(r0 / G, T - 1);
    const int nsafe = min(max(len - (T - 1 - t_first) - k0, 0), nkeys);
    const int64_t base = (((int64_t)b * Hkv + h) * U + k0) * row_bytes<MOSKA_BF16>();
    WaveState<NR> st;
    attend<NR, MOSKA_BF16, NW, AUX, NKB>(st, qf, (const char *)a.Ku + base, (const char *)a.Vu + base, nkeys, nsafe, lim,
                                         scale * kLog2e, wave, q, x);
    combine_and_store<NR, NW, !SPLIT>(st, comb, threadIdx.x, wave, q, x, orow, 1.f, SPLIT ? a.split_O : a.part_O,
                                      SPLIT ? a.split_LSE : a.part_LSE);
}

}  // namespace mfma
}  // namespace moska
