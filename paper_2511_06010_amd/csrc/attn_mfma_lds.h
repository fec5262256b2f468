// Shared KV Attention on LDS-staged tiles of 64, 128 or 256 query rows (smaller row counts pad a
// 64-row tile), paper Sec. III-A: the regime where batching the queries of a chunk turns the chunk's
// K/V stream into a GEMM.
//
// A workgroup of NWV waves owns 16*NR*NWV rows of one bucket; each wave owns NR blocks of 16 of them
// (blocks w, w + NWV, ... of wave w) for ALL keys of the chunk, so no cross-wave merge is needed.  The chunk's K and V are streamed
// from HBM once per workgroup: every thread fetches a slice of the next KT-key stage into
// registers while the current stage is consumed from LDS, then writes its slice to the other
// LDS buffer.  One barrier per stage.  lds_tile serves a bf16 store; lds_tile_f8 an fp8 store, whose
// keys stay fp8 in LDS for the scaled fp8 MFMA while its values are widened to bf16 on the way in
// (once per workgroup, not once per wave); shared_all_kernel / shared_small_kernel / shared_light_f8_kernel
// are the launches.
//
// LDS stage layout (bf16): K[keys][256 B] with the 16-byte units of a row XOR-swizzled by
// (key & 15), so the MFMA A-operand read (16 keys x one unit, 16 lanes per phase) is free of bank
// conflicts; V[keys][256 B] with the 32-byte dim blocks of a row XOR-swizzled by (key & 7) for the
// transpose read that builds the V^T operand without any register shuffling.  Scores and softmax
// reuse the code of the streaming kernels (attn_mfma.h).
#pragma once

#include <type_traits>

#include "attn_mfma.h"

namespace moska {
namespace mfma {

// One thread's slice of a KT-key stage in registers (T threads per workgroup).
template <int KVD, int T, int KT> struct StageRegs {
    // 16-byte units of K (and of V) per thread; a unit of fp8 becomes two units of bf16 in LDS
    static constexpr int N = (KT * (KVD == MOSKA_BF16 ? 16 : 8)) / T;
    static_assert(N >= 1, "stage too small for the workgroup");
    uint4 k[N], v[N];
};

template <int KVD, int T, int KT, int AUX>
__device__ __forceinline__ void stage_fetch(StageRegs<KVD, T, KT> &r, __amdgpu_buffer_rsrc_t rk,
                                            __amdgpu_buffer_rsrc_t rv, int stage, int tid) {
    constexpr int ROWB = row_bytes<KVD>();
    constexpr int N = StageRegs<KVD, T, KT>::N;
    const uint32_t off = (uint32_t)stage * (KT * ROWB) + (uint32_t)tid * 16u;   // consecutive threads, consecutive units
#pragma unroll
    for (int i = 0; i < N; ++i) {
        r.k[i] = as_uint4(__builtin_amdgcn_raw_buffer_load_b128(rk, off + i * T * 16, 0, AUX));
        r.v[i] = as_uint4(__builtin_amdgcn_raw_buffer_load_b128(rv, off + i * T * 16, 0, AUX));
    }
}

__device__ __forceinline__ void fp8x16_to_bf16(const uint4 &w, uint4 &lo, uint4 &hi) {
    fp8x4_to_bf16x4(w.x, lo.x, lo.y);
    fp8x4_to_bf16x4(w.y, lo.z, lo.w);
    fp8x4_to_bf16x4(w.z, hi.x, hi.y);
    fp8x4_to_bf16x4(w.w, hi.z, hi.w);
}

// lk, lv: one LDS buffer's K and V areas (KT*16 uint4 each)
template <int KVD, int T, int KT>
__device__ __forceinline__ void stage_store(const StageRegs<KVD, T, KT> &r, uint4 *lk, uint4 *lv, int tid) {
    constexpr int N = StageRegs<KVD, T, KT>::N;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int g = tid + i * T;
        static_assert(KVD == MOSKA_BF16, "an fp8 store is staged by lds_tile_f8");
        const int row = g >> 4, u = g & 15;
        lk[row * 16 + (u ^ (row & 15))] = r.k[i];
        lv[row * 16 + ((((u >> 1) ^ (row & 7)) << 1) | (u & 1))] = r.v[i];
    }
}

// S^T of one 32-key sub-tile with the key operands read from LDS one 16-key block at a time
// (lane layout as in the streaming kernels; the XOR swizzle makes the reads conflict free)
template <int NR, int NA = NR>
__device__ __forceinline__ void qk_from_lds(f32x4 (&s)[NR][2], const uint32_t (&qf)[NR][4][4], const uint4 *lk, int q,
                                            int x) {
#pragma unroll
    for (int kblk = 0; kblk < 2; ++kblk) {
        uint32_t kf[4][4];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            const uint4 v = lk[(16 * kblk + x) * 16 + ((4 * kb + q) ^ x)];
            kf[kb][0] = v.x; kf[kb][1] = v.y; kf[kb][2] = v.z; kf[kb][3] = v.w;
        }
#pragma unroll
        for (int rb = 0; rb < NA; ++rb) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) acc = mfma16(kf[kb], qf[rb][kb], acc);
            s[rb][kblk] = acc;
        }
    }
}

// O^T += V^T P^T of one 32-key sub-tile with the V^T operand fetched by the LDS transpose read
// (ds_read_b64_tr_b16): inside a 16-lane group, source lane S reads four consecutive dims of key
// row S/4 and result lane x receives dim x of the four rows -- exactly the MFMA A operand
// (dim x of 4 key slots).  MFMA e covers dims 16e..16e+15, so component r of o[rb][e] is dim
// 16e + 4q + r.  The 32-byte dim blocks of a value row are XOR-swizzled by (key & 7): the 16 keys
// of a read land on 8 different blocks (measured: 2 cycles an instruction, no bank conflicts).
template <int NR, int NA = NR>
__device__ __forceinline__ void pv_from_lds(WaveState<NR> &st, const uint4 *lv, const uint32_t (&pf)[NR][4], int lane) {
    typedef __attribute__((ext_vector_type(4))) short s16x4;
    typedef __attribute__((address_space(3))) s16x4 *lds_s16x4;
    const int q = lane >> 4, S = lane & 15;
    const int key = 4 * q + (S >> 2);                       // and key + 16 for slots 4..7
    const char *rowp = (const char *)lv + key * 256 + (S & 3) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const char *p = rowp + ((e ^ (key & 7)) << 5);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(p + 16 * 256));
        const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
        const uint32_t vf[4] = {l2.x, l2.y, h2.x, h2.y};
#pragma unroll
        for (int rb = 0; rb < NA; ++rb) st.o[rb][e] = mfma16(vf, pf[rb], st.o[rb][e]);
    }
}

// LDS footprint of a tile kernel, in uint4 units: two buffers of K and V stages
template <int KT> constexpr int lds_units() { return 4 * KT * 16; }

// Tile (bkt, row0) on the LDS-staged path: 16*NR*NWV rows, by the NWV*64 threads tid = 0 .. NWV*64-1
// that share smem (lds_units<KT>() uint4).  Contains one workgroup barrier per stage plus one.
// KT keys per stage (32 or 64); PD stages of global loads are kept in flight in registers (1, 2 or 4):
// the loads of stage t+1+PD are issued when stage t+1 has been copied to LDS, so they have PD
// stages of MFMA work to land.
template <int NR, int NWV, int KVD, int AUX, int KT, int PD, bool SPLIT>
__device__ __forceinline__ void lds_tile(const SharedArgs &a, int bkt, int row0, int Hq, int Hkv, int C, int Lchunk,
                                         int k, float scale, uint4 *smem, int tid) {
    static_assert(KT == 32 || KT == 64 || KT == 128, "keys per stage");
    static_assert(PD == 1 || PD == 2 || PD == 4, "stages in flight");
    constexpr int T = NWV * 64;
    constexpr int SU = KT * 16;                            // uint4 units of K (or V) per stage
    uint4 *ldsK = smem, *ldsV = smem + 2 * SU;
    const int h = bkt / C, c = bkt - h * C, G = Hq / Hkv;
    const int lane = tid & 63, q = lane >> 4, x = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // this workgroup's keys: L of them from first_key on (the whole chunk unless chunks are split over
    // workgroups).  Their first stage is requested before anything else: the bucket -> item -> query row
    // chain below is three dependent loads, a long time to have nothing else in flight.
    int first_key, L;
    key_slice(Lchunk, a.nsplit, blockIdx.y, KT, first_key, L);
    const int64_t base = (((int64_t)c * Hkv + h) * Lchunk + first_key) * row_bytes<KVD>();
    const __amdgpu_buffer_rsrc_t rk = key_set_rsrc((const char *)a.Ks + base, (uint32_t)L * row_bytes<KVD>());
    const __amdgpu_buffer_rsrc_t rv = key_set_rsrc((const char *)a.Vs + base, (uint32_t)L * row_bytes<KVD>());
    const int nst = (L + KT - 1) / KT;                     // stages; rows past L read as zeros
    StageRegs<KVD, T, KT> regs[PD];                        // PD >= 2: regs[(t+1+j) % PD] carries stage t+1+j at step t
    stage_fetch<KVD, T, KT, AUX>(regs[0], rk, rv, 0, tid);

    const int beg = a.off[bkt], rows = (a.off[bkt + 1] - beg) * G;
    uint32_t qf[NR][4][4];
    int64_t orow[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int rr = row0 + (rb * NWV + wave) * 16 + x;   // row blocks are dealt to the waves round-robin
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
        load_q<MOSKA_BF16>(qf[rb], a.Q, qoff, valid, q);    // keys sit in LDS as bf16 in natural dim order
    }
    const float kmul = a.scale_k ? a.scale_k[c * Hkv + h] : 1.f;
    const float vmul = a.scale_v ? a.scale_v[c * Hkv + h] : 1.f;
    const float sc = scale * kmul * kLog2e;

    WaveState<NR> st;
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        st.m[rb] = -INFINITY;
        st.l[rb] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[rb][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Row block rb * NWV + wave is the wave's block rb: a tile that is not full leaves every SIMD about the same
    // number of blocks (the two waves of a SIMD in a 256-row tile are waves w and w + 4).  A wave whose second block
    // lies past the bucket's end works on one block; a wave without rows only helps to stage K and V.
    const int nblk = __builtin_amdgcn_readfirstlane((rows - row0 + 15) >> 4);
    const bool has_rows = wave < nblk, two = NR == 2 && NWV + wave < nblk;
    // stage t out of LDS buffer `cur`: scores, softmax, output for its 32-key sub-tiles, on NA row blocks
    auto consume_n = [&](auto na, int t, int cur) {
        constexpr int NA = decltype(na)::value;
#pragma unroll
        for (int sub = 0; sub < KT / 32; ++sub) {
            f32x4 s[NR][2];
            uint32_t pf[NR][4];
            const int key0 = KT * t + 32 * sub;
            qk_from_lds<NR, NA>(s, qf, ldsK + cur * SU + sub * 512, q, x);
            if (key0 + 32 > L) softmax_tile<NR, true, NA>(st, s, pf, key0, L, sc, q);
            else softmax_tile<NR, false, NA>(st, s, pf, key0, L, sc, q);
            pv_from_lds<NR, NA>(st, ldsV + cur * SU + sub * 512, pf, lane);
        }
    };
    stage_store<KVD, T, KT>(regs[0], ldsK, ldsV, tid);
    // the stage loop, once per number of row blocks the wave works on (0: staging only); every form
    // executes the same barriers
    auto run = [&](auto na) {
        auto consume = [&](int t, int cur) {
            if constexpr (decltype(na)::value > 0) consume_n(na, t, cur);
        };
        if constexpr (PD == 1) {
            __syncthreads();
            for (int t = 0; t < nst; ++t) {
                const int cur = t & 1;
                stage_fetch<KVD, T, KT, AUX>(regs[0], rk, rv, t + 1, tid);   // past the end: dropped by the range check
                consume(t, cur);
                stage_store<KVD, T, KT>(regs[0], ldsK + (cur ^ 1) * SU, ldsV + (cur ^ 1) * SU, tid);
                __syncthreads();
            }
        } else {
#pragma unroll
            for (int j = 0; j < PD; ++j) stage_fetch<KVD, T, KT, AUX>(regs[(1 + j) % PD], rk, rv, 1 + j, tid);
            __syncthreads();
            for (int t0 = 0; t0 < nst; t0 += PD) {
#pragma unroll
                for (int u = 0; u < PD; ++u) {             // unrolled: buffer and register indices are constants
                    const int t = t0 + u;
                    if (t < nst) {
                        consume(t, u & 1);
                        StageRegs<KVD, T, KT> &nx = regs[(u + 1) % PD];   // the registers that carry stage t+1
                        stage_store<KVD, T, KT>(nx, ldsK + ((u + 1) & 1) * SU, ldsV + ((u + 1) & 1) * SU, tid);
                        stage_fetch<KVD, T, KT, AUX>(nx, rk, rv, t + 1 + PD, tid);
                        __syncthreads();
                    }
                }
            }
        }
    };
    if (NR == 1 ? has_rows : two) run(std::integral_constant<int, NR>{});
    else if (NR == 2 && has_rows) run(std::integral_constant<int, 1>{});
    else run(std::integral_constant<int, 0>{});
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        st.l[rb] = row_lanes_sum(st.l[rb]);
    }
    store_rows<NR, !SPLIT>(st, q, orow, vmul, SPLIT ? a.split_O : a.part_O, SPLIT ? a.split_LSE : a.part_LSE);
}

// ---- fp8 store: scores on the fp8 matrix cores --------------------------------------------------
//
// v_mfma_scale_f32_16x16x128_f8f6f4 contracts all 128 head dims of 16 keys x 16 query rows in one
// instruction, at twice the rate of the bf16 MFMA, from e4m3 operands with a power-of-two scale
// per row.  The keys of an fp8 store are its A operand as they are: they stay fp8 in LDS (half the
// stage bytes and half the LDS read traffic of the bf16 stage, no widening).  The query row has no
// fp8 twin, so it is carried as a pair hi + lo of e4m3 values (hi = the row rounded to e4m3 after
// scaling its largest element into [128, 256), lo = the rounding error, again in e4m3): together
// 8 significant bits, the precision of the bf16 query itself, for two MFMAs at the doubled rate --
// the cost of the bf16 contraction.  The logit scale, the keys' dequantisation factor and log2(e)
// are folded into the query before the split, and the running reference point m of the softmax row
// enters as the accumulator's initial value, so the MFMA hands the softmax s*log2(e) - m directly
// and the per-score scale-and-subtract disappears from the vector ALU.
// Operand layout (measured): lane (q,x) holds 32 bytes of row x; the instruction pairs A and B
// bytes position by position, so any 32 dims may sit there as long as both operands agree; the
// block scales of a row are taken from the scale registers of the row's four lanes, which hold
// one common value here.
typedef __attribute__((ext_vector_type(8))) int i32x8;
// The 256-row tile of an fp8 store takes stages of 128 keys (96 KiB of LDS: half as many barriers; +4 % at 4096
// rows per bucket) with one stage of loads in flight; for a bf16 store 128-key stages fill all 128 KiB and measured
// 25 % slower, so it stays at 64 keys with two stages in flight.
#ifndef MOSKA_BIG_KT
#define MOSKA_BIG_KT 128
#endif
#ifndef MOSKA_BIG_PD
#define MOSKA_BIG_PD 1
#endif

__device__ __forceinline__ f32x4 mfma_f8(const i32x8 &a, const i32x8 &b, f32x4 c, int scale_b) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 0, 0, 0x7F7F7F7F, 0, scale_b);
}

struct QueryF8 {
    i32x8 hi, lo;       // dims 32q .. 32q+31 of the scaled row, and the rounding error of hi
    int scale;          // e8m0 exponent byte (replicated) that undoes the row's scaling
};

// Row at element offset qoff of Q (bf16), times c, as an fp8 pair; a padding row (valid = false) is zero.
__device__ __forceinline__ void load_q_f8(QueryF8 &qf, const void *Q, int64_t qoff, bool valid, float c, int q) {
    float xv[32];
    float amax = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint4 v = {0u, 0u, 0u, 0u};
        if (valid) v = *(const uint4 *)((const uint16_t *)Q + qoff + 32 * q + 8 * u);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            xv[8 * u + 2 * i] = bf16_bits_to_f32(w[i] & 0xFFFFu) * c;
            xv[8 * u + 2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u) * c;
        }
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(xv[i]));
    amax = row_lanes_max(amax);                             // over the row's 128 dims
    int e = amax > 0.f ? __builtin_amdgcn_frexp_expf(amax) : 0;   // amax = f * 2^e, f in [0.5, 1)
    int sh = 8 - e;                                         // largest element lands in [128, 256)
    sh = sh > 100 ? 100 : sh < -100 ? -100 : sh;
    const int sb = 127 - sh;                                // the MFMA multiplies the row by 2^(sb - 127)
    qf.scale = sb | (sb << 8) | (sb << 16) | (sb << 24);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float y[4], r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = __builtin_ldexpf(xv[4 * i + j], sh);
        int h = 0;
        h = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], h, false);
        h = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], h, true);
        const f32x2 b0 = __builtin_amdgcn_cvt_pk_f32_fp8(h, false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8(h, true);
        r[0] = y[0] - b0[0]; r[1] = y[1] - b0[1]; r[2] = y[2] - b1[0]; r[3] = y[3] - b1[1];
        int l = 0;
        l = __builtin_amdgcn_cvt_pk_fp8_f32(r[0], r[1], l, false);
        l = __builtin_amdgcn_cvt_pk_fp8_f32(r[2], r[3], l, true);
        qf.hi[i] = h;
        qf.lo[i] = l;
    }
}

// XOR swizzle of the eight 16-byte units of an fp8 key row in LDS.  A 128-bit LDS read is served 16 lanes a
// cycle over 64 banks, and the 16 lanes are not consecutive (measured with a two-lane probe and the bank-conflict
// counter): lanes {0-3, 12-15, 20-23, 24-27} go together, {4-11, 16-19, 28-31} likewise, and the same in the
// upper half of the wave.  In the score read below that is keys {0-3, 12-15} of one q together with keys 4-11 of
// the next q, whose units differ by 2: the swizzle sends the first key set to units 0-3 (xor the unit read) and
// the second to units 4-7, separately for the even and the odd key of each 256-byte line, so a cycle's 16 pieces
// fall into 16 different bank groups.  (With key & 7 as the swizzle every such read took 8 cycles instead of 4.)
__device__ __forceinline__ int f8_key_swizzle(int key) { return ((key + 4) >> 1) & 7; }

// t = s*log2(e) - m of one 32-key sub-tile: the key operands (fp8, 16-byte units of a 128-byte row
// XOR-swizzled by f8_key_swizzle) from LDS, the accumulators starting at -m of the lane's row.
template <int NR, int NA = NR>
__device__ __forceinline__ void qk_from_lds_f8(f32x4 (&t)[NR][2], const QueryF8 (&qf)[NR], const f32x4 (&negm)[NR],
                                               const uint4 *lk, int q, int x) {
#pragma unroll
    for (int kblk = 0; kblk < 2; ++kblk) {
        const int row = 16 * kblk + x, sw = f8_key_swizzle(x);
        const uint4 u0 = lk[row * 8 + ((2 * q) ^ sw)], u1 = lk[row * 8 + ((2 * q + 1) ^ sw)];
        const i32x8 kf = {(int)u0.x, (int)u0.y, (int)u0.z, (int)u0.w, (int)u1.x, (int)u1.y, (int)u1.z, (int)u1.w};
#pragma unroll
        for (int rb = 0; rb < NA; ++rb) {
            const f32x4 acc = mfma_f8(kf, qf[rb].hi, negm[rb], qf[rb].scale);
            t[rb][kblk] = mfma_f8(kf, qf[rb].lo, acc, qf[rb].scale);
        }
    }
}

// Online softmax on scores that arrive with the row's reference point already subtracted (log2
// domain).  The reference moves only when a tile's maximum exceeds it by more than kLazy -- and at
// the row's first tile (`first`, wave-uniform), where it moves onto the tile's maximum from its
// starting value 0; only then are the scores corrected by the move.
// negm: -m of the lane's row in all four components, the accumulator start of the next scores.
template <int NR, bool TAIL, int NA = NR>
__device__ __forceinline__ void softmax_presub(WaveState<NR> &st, f32x4 (&negm)[NR], const f32x4 (&t)[NR][2],
                                               uint32_t (&pf)[NR][4], int key0, int nkeys, int q, bool first) {
    float v[NR][8], mx[NR];
    bool over = first;
#pragma unroll
    for (int rb = 0; rb < NA; ++rb) {
#pragma unroll
        for (int kblk = 0; kblk < 2; ++kblk)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float z = t[rb][kblk][r];
                if (TAIL && key0 + 16 * kblk + 4 * q + r >= nkeys) z = -INFINITY;   // rows past the end read as 0
                v[rb][4 * kblk + r] = z;
            }
        const float *w = v[rb];
        mx[rb] = fmaxf(fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3])), fmaxf(fmaxf(w[4], w[5]), fmaxf(w[6], w[7])));
        over |= mx[rb] > kLazy;
    }
    if (__any(over)) {
        float alpha[NR];
#pragma unroll
        for (int rb = 0; rb < NA; ++rb) {
            const float rmx = row_lanes_max(mx[rb]);
            const float delta = (first || rmx > kLazy) ? rmx : 0.f;     // finite: a tile holds a key of every row
            alpha[rb] = __builtin_amdgcn_exp2f(-delta);
            st.m[rb] += delta;
            negm[rb] = f32x4{-st.m[rb], -st.m[rb], -st.m[rb], -st.m[rb]};
            st.l[rb] *= alpha[rb];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[rb][i] -= delta;
        }
#pragma unroll
        for (int rb = 0; rb < NA; ++rb)
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int r = 0; r < 4; ++r) st.o[rb][e][r] *= alpha[rb];
    }
#pragma unroll
    for (int rb = 0; rb < NA; ++rb) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[rb][i] = __builtin_amdgcn_exp2f(v[rb][i]);
        pf[rb][0] = pack_bf16(v[rb][0], v[rb][1]);
        pf[rb][1] = pack_bf16(v[rb][2], v[rb][3]);
        pf[rb][2] = pack_bf16(v[rb][4], v[rb][5]);
        pf[rb][3] = pack_bf16(v[rb][6], v[rb][7]);
#pragma unroll
        for (int i = 0; i < 4; ++i) st.l[rb] = dot2_ones(pf[rb][i], st.l[rb]);
    }
}

// LDS of the fp8 tile, in uint4 units: two buffers of KT-key stages, keys as fp8 (8 units a key), values as bf16 (16)
constexpr int lds_units_f8(int KT) { return 2 * KT * 8 + 2 * KT * 16; }

// Tile (bkt, row0) of an fp8 store on the LDS-staged path with fp8 scores: 16*NR*NWV rows, by the
// NWV*64 threads tid = 0 .. NWV*64-1 that share smem (two buffers of KT keys x 8 uint4 and of KT values x 16
// uint4); stages of KT = 64 or 128 keys, PD (1, 2 or 4) stages of global loads in flight.  One workgroup barrier per stage plus one, as lds_tile.
template <int NR, int NWV, int AUX, int PD, bool SPLIT, int KT = 64>
__device__ __forceinline__ void lds_tile_f8(const SharedArgs &a, int bkt, int row0, int Hq, int Hkv, int C, int Lchunk,
                                            int k, float scale, uint4 *smem, int tid) {
    static_assert(PD == 1 || PD == 2 || PD == 4, "stages in flight");
    static_assert(KT == 64 || KT == 128, "keys per stage");
    static_assert(lds_units_f8(KT) <= (NWV == 8 ? 2 : 1) * lds_units<64>(), "a half workgroup has 64 KiB, a whole one 128");
    constexpr int KVD = MOSKA_FP8_E4M3, T = NWV * 64;
    constexpr int KU = KT * 8, VU = KT * 16;                // uint4 units of a K stage and of a V stage
    uint4 *ldsK = smem, *ldsV = smem + 2 * KU;
    const int h = bkt / C, c = bkt - h * C, G = Hq / Hkv;
    const int lane = tid & 63, q = lane >> 4, x = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int first_key, L;
    key_slice(Lchunk, a.nsplit, blockIdx.y, KT, first_key, L);
    const int64_t base = (((int64_t)c * Hkv + h) * Lchunk + first_key) * row_bytes<KVD>();
    const __amdgpu_buffer_rsrc_t rk = key_set_rsrc((const char *)a.Ks + base, (uint32_t)L * row_bytes<KVD>());
    const __amdgpu_buffer_rsrc_t rv = key_set_rsrc((const char *)a.Vs + base, (uint32_t)L * row_bytes<KVD>());
    const int nst = (L + KT - 1) / KT;
    StageRegs<KVD, T, KT> regs[PD];
    stage_fetch<KVD, T, KT, AUX>(regs[0], rk, rv, 0, tid);

    const float kmul = a.scale_k[c * Hkv + h], vmul = a.scale_v[c * Hkv + h];
    const int beg = a.off[bkt], rows = (a.off[bkt + 1] - beg) * G;
    QueryF8 qf[NR];
    int64_t orow[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int rr = row0 + (rb * NWV + wave) * 16 + x;   // row blocks are dealt to the waves round-robin
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
        load_q_f8(qf[rb], a.Q, qoff, valid, scale * kmul * kLog2e, q);
    }

    WaveState<NR> st;
    f32x4 negm[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        st.m[rb] = 0.f;                                     // moved onto the first tile's maximum by softmax_presub
        negm[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.l[rb] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[rb][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // row block rb * NWV + wave is the wave's block rb, as in lds_tile: one or two blocks of work per wave
    const int nblk = __builtin_amdgcn_readfirstlane((rows - row0 + 15) >> 4);
    const bool has_rows = wave < nblk, two = NR == 2 && NWV + wave < nblk;
    auto consume_n = [&](auto na, int t, int cur) {
        constexpr int NA = decltype(na)::value;
#pragma unroll
        for (int sub = 0; sub < KT / 32; ++sub) {
            f32x4 s[NR][2];
            uint32_t pf[NR][4];
            const int key0 = KT * t + 32 * sub;
            qk_from_lds_f8<NR, NA>(s, qf, negm, ldsK + cur * KU + sub * 256, q, x);
            if (key0 + 32 > L) softmax_presub<NR, true, NA>(st, negm, s, pf, key0, L, q, key0 == 0);
            else softmax_presub<NR, false, NA>(st, negm, s, pf, key0, L, q, key0 == 0);
            pv_from_lds<NR, NA>(st, ldsV + cur * VU + sub * 512, pf, lane);
        }
    };
    auto store = [&](const StageRegs<KVD, T, KT> &r, int buf) {
        uint4 *lk = ldsK + buf * KU, *lv = ldsV + buf * VU;
#pragma unroll
        for (int i = 0; i < StageRegs<KVD, T, KT>::N; ++i) {
            const int g = tid + i * T, row = g >> 3, u = g & 7;
            lk[row * 8 + (u ^ f8_key_swizzle(row))] = r.k[i];   // keys stay fp8
            uint4 lo, hi;
            fp8x16_to_bf16(r.v[i], lo, hi);                 // values are widened for the bf16 P V product
            // (a 128-bit LDS write is served 8 consecutive lanes a cycle over 128 bytes of banks, so the low
            // halves of a row's 8 blocks collide in pairs: 16 cycles an instruction instead of 8.  Storing the
            // halves of blocks 4-7 the other way round removes that and measured 1 % slower in the kernel.)
            const int vb = (u ^ (row & 7)) * 2;
            lv[row * 16 + vb] = lo;
            lv[row * 16 + vb + 1] = hi;
        }
    };
    store(regs[0], 0);
    // the stage loop, once per number of row blocks the wave works on (0: staging only), as in lds_tile
    auto run = [&](auto na) {
        auto consume = [&](int t, int cur) {
            if constexpr (decltype(na)::value > 0) consume_n(na, t, cur);
        };
        if constexpr (PD == 1) {
            __syncthreads();
            for (int t = 0; t < nst; ++t) {
                const int cur = t & 1;
                stage_fetch<KVD, T, KT, AUX>(regs[0], rk, rv, t + 1, tid);
                consume(t, cur);
                store(regs[0], cur ^ 1);
                __syncthreads();
            }
        } else {
#pragma unroll
            for (int j = 0; j < PD; ++j) stage_fetch<KVD, T, KT, AUX>(regs[(1 + j) % PD], rk, rv, 1 + j, tid);
            __syncthreads();
            for (int t0 = 0; t0 < nst; t0 += PD) {
#pragma unroll
                for (int u = 0; u < PD; ++u) {
                    const int t = t0 + u;
                    if (t < nst) {
                        consume(t, u & 1);
                        StageRegs<KVD, T, KT> &nx = regs[(u + 1) % PD];
                        store(nx, (u + 1) & 1);
                        stage_fetch<KVD, T, KT, AUX>(nx, rk, rv, t + 1 + PD, tid);
                        __syncthreads();
                    }
                }
            }
        }
    };
    if (NR == 1 ? has_rows : two) run(std::integral_constant<int, NR>{});
    else if (NR == 2 && has_rows) run(std::integral_constant<int, 1>{});
    else run(std::integral_constant<int, 0>{});
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) st.l[rb] = row_lanes_sum(st.l[rb]);
    store_rows<NR, !SPLIT>(st, q, orow, vmul, SPLIT ? a.split_O : a.part_O, SPLIT ? a.split_LSE : a.part_LSE);
}

// A tile of up to 128 rows on the LDS-staged path, by the 256 threads tid = 0 .. 255 that share sm
// (64 KiB): 4 waves x 16 rows (up to 64 rows) or 4 waves x 32 rows.  One stage of loads in flight:
// two or four measured the same to within 2 % for either store (these tiles are bound by what a
// compute unit gets done per stage, not by the latency of its loads).
#ifndef MOSKA_PD_F8
#define MOSKA_PD_F8 1
#endif
#ifndef MOSKA_PD_B16
#define MOSKA_PD_B16 1
#endif
template <int KVD, int AUX, bool SPLIT>
__device__ __forceinline__ void staged_small_tile(const SharedArgs &a, bool rows128, int bkt, int row0, int Hq, int Hkv,
                                                  int C, int L, int k, float scale, uint4 *sm, int tid) {
    if constexpr (KVD == MOSKA_FP8_E4M3) {
        if (rows128) lds_tile_f8<2, 4, AUX, MOSKA_PD_F8, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, sm, tid);
        else lds_tile_f8<1, 4, AUX, MOSKA_PD_F8, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, sm, tid);
    } else {
        if (rows128) lds_tile<2, 4, KVD, AUX, 64, MOSKA_PD_B16, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, sm, tid);
        else lds_tile<1, 4, KVD, AUX, 64, MOSKA_PD_B16, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, sm, tid);
    }
}

// The tile list in ONE launch of 512-thread workgroups (pairs != 0), so that no size class pays a
// kernel's fill and drain of its own and the long 256-row tiles run beside the streaming ones; or
// only its 256-row tiles (pairs == 0), the others going to shared_small_kernel.  Three kinds of
// work item:
//   256-row tile        one per workgroup (8 waves x 32 rows)
//   staged pair         two LDS-staged tiles of up to 128 rows per workgroup, one per half (4 waves
//                       each, with its own half of the LDS); both halves stream chunks of the same
//                       length, so they execute the same number of workgroup barriers
//   streaming pair      (fp8 store) two streaming tiles of up to 32 rows, one per half: an fp8 store
//                       streams them (each wave its own keys, twice the bytes in flight of an fp8 LDS
//                       stage); a bf16 store is faster through LDS like the 64-row tiles
// The grid is sized on the host from upper bounds; workgroups beyond the items that exist return.
// A half without a tile of its own repeats its sibling's (same values to the same slots).
template <int KVD, int AUX, bool SPLIT>
__global__ __launch_bounds__(512, 2) void shared_all_kernel(SharedArgs a, int pairs, int Hq, int Hkv, int C,
                                                             int L, int k, float scale) {
    constexpr int HALF = lds_units<64>();                   // 64 KiB of K/V stages, or a 33 KiB merge buffer
    __shared__ uint4 smem[2 * HALF];
    static_assert(sizeof(uint4) * HALF >= sizeof(float) * 2 * 32 * OSTRIDE, "merge buffer of the 32-row streaming path");
    constexpr int S0 = KVD == MOSKA_FP8_E4M3 ? 2 : 0;        // first class of the LDS-staged small tiles
    // work items: 256-row tiles, pairs of LDS-staged small tiles, pairs of streaming tiles; each XCD
    // (workgroups are dealt to the 8 XCDs round-robin) takes a contiguous share of each list, so that
    // the tiles of one bucket, which re-read the same chunk, share an L2
    const int n4 = a.tile_hdr[5] - a.tile_hdr[4], nL = a.tile_hdr[4] - a.tile_hdr[S0], nS = a.tile_hdr[S0] - a.tile_hdr[0];
    const int p4 = (n4 + 7) >> 3, pL = pairs ? (((nL + 1) >> 1) + 7) >> 3 : 0, pS = pairs ? (((nS + 1) >> 1) + 7) >> 3 : 0;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per = p4 + pL + pS;
    if (slot >= per) return;
    // slot -> (kind, index inside the XCD's share): the long 256-row tiles first.  (Spreading them
    // evenly among the others, or putting them last, measured the same to within 3 %.)
    if (slot < p4) {
        const int w = xcd * p4 + slot;
        if (w >= n4) return;
        const int t = a.tile_hdr[4] + w;
        if constexpr (KVD == MOSKA_FP8_E4M3)
            lds_tile_f8<2, 8, AUX, MOSKA_BIG_PD, SPLIT, MOSKA_BIG_KT>(a, a.tiles[2 * t], a.tiles[2 * t + 1], Hq, Hkv, C, L, k, scale, smem, threadIdx.x);
        else
            lds_tile<2, 8, KVD, AUX, 64, 2, SPLIT>(a, a.tiles[2 * t], a.tiles[2 * t + 1], Hq, Hkv, C, L, k, scale, smem,
                                                   threadIdx.x);
        return;
    }
    int r = slot - p4;                                      // index among the XCD's pairs: staged ones first
    const int half = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8), tid = threadIdx.x & 255;
    uint4 *sm = smem + half * HALF;
    const bool staged = r < pL;
    if (!staged) r -= pL;
    const int n = staged ? nL : nS, w = xcd * (staged ? pL : pS) + r;
    if (2 * w >= n) return;
    const int i = 2 * w + half < n ? 2 * w + half : 2 * w;
    const int t = a.tile_hdr[staged ? 4 : S0] - 1 - i;      // each list is walked from its end: largest tiles first
    const int bkt = a.tiles[2 * t], row0 = a.tiles[2 * t + 1];
    if (staged) {
        staged_small_tile<KVD, AUX, SPLIT>(a, t >= a.tile_hdr[3], bkt, row0, Hq, Hkv, C, L, k, scale, sm, tid);
    } else if constexpr (S0 > 0) {
        if (t >= a.tile_hdr[1]) stream_tile<2, KVD, 4, AUX, 1, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, (float *)sm, tid);
        else stream_tile<1, KVD, 4, AUX, 1, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, (float *)sm, tid);
    }
}

// The tiles of classes c_lo .. 3 (up to 128 rows), one per 256-thread workgroup (two workgroups share a
// compute unit and run independently of each other).
template <int KVD, int AUX, bool SPLIT>
__global__ __launch_bounds__(256, 2) void shared_small_kernel(SharedArgs a, int c_lo, int Hq, int Hkv, int C, int L,
                                                               int k, float scale) {
    __shared__ uint4 sm[lds_units<64>()];
    constexpr int S0 = KVD == MOSKA_FP8_E4M3 ? 2 : 0;
    const int n = a.tile_hdr[4] - a.tile_hdr[c_lo];
    const int w = xcd_tile_index(blockIdx.x, n);
    if (w < 0) return;
    const int t = a.tile_hdr[4] - 1 - w;                    // walked from the end: largest tiles first
    const int bkt = a.tiles[2 * t], row0 = a.tiles[2 * t + 1], tid = threadIdx.x;
    if (t >= a.tile_hdr[S0]) {
        staged_small_tile<KVD, AUX, SPLIT>(a, t >= a.tile_hdr[3], bkt, row0, Hq, Hkv, C, L, k, scale, sm, tid);
    } else if constexpr (S0 > 0) {
        if (t >= a.tile_hdr[1]) stream_tile<2, KVD, 4, AUX, 1, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, (float *)sm, tid);
        else stream_tile<1, KVD, 4, AUX, 1, SPLIT>(a, bkt, row0, Hq, Hkv, C, L, k, scale, (float *)sm, tid);
    }
}

// The tiles of an fp8 store of up to 64 rows, one per 256-thread workgroup, all on the LDS-staged path (4 waves
// x 16 rows; waves without rows help staging).  Without the 128-row tile's 32 rows per wave the code needs under
// 168 registers and 48 KiB of LDS, so three workgroups share a compute unit: 12 waves instead of 8 to cover each
// other's barriers and load waits.  Measured on 1024 chunks x 4096 tokens, top-256: 7-12 % faster at 16-64 rows
// per bucket than two workgroups per compute unit with the 16- and 32-row tiles streaming; streaming tiles in
// this kernel (a few registers spilled) are slower than either.  (A bf16 store's tiles would need 32-key stages
// to fit three or four workgroups: measured no faster with 64-128 rows per bucket and 15-45 % slower below.)
template <int AUX, bool SPLIT>
__global__ __launch_bounds__(256, 3) void shared_light_f8_kernel(SharedArgs a, int Hq, int Hkv, int C, int L, int k,
                                                                  float scale) {
    __shared__ uint4 sm[lds_units_f8(64)];
    const int n = a.tile_hdr[3] - a.tile_hdr[0];
    const int w = xcd_tile_index(blockIdx.x, n);
    if (w < 0) return;
    const int t = a.tile_hdr[3] - 1 - w;                    // walked from the end: largest tiles first
    lds_tile_f8<1, 4, AUX, MOSKA_PD_F8, SPLIT>(a, a.tiles[2 * t], a.tiles[2 * t + 1], Hq, Hkv, C, L, k, scale, sm,
                                               threadIdx.x);
}

}  // namespace mfma
}  // namespace moska
