// Launcher of the MFMA Shared KV Attention for one key/value dtype; included by one translation
// unit per dtype so the instantiations compile in parallel.
#pragma once

#include "attn_mfma_lds.h"

namespace moska {
namespace mfma {

// shared_all_kernel serves the 256-row tiles and, when the small tiles go in pairs, those too:
// workgroups for the 256-row tiles, for pairs of LDS-staged small tiles and, for an fp8 store, for
// pairs of streaming tiles, each count taken from the host-side bound on the tiles of that kind and
// rounded up to a multiple of 8.  Otherwise the small tiles follow in shared_small_kernel (an fp8
// store's tiles of up to 64 rows in shared_light_f8_kernel when there are many buckets).
template <int KVD>
int launch_shared_classes(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    constexpr int S0 = KVD == MOSKA_FP8_E4M3 ? 2 : 0;       // first class of the LDS-staged small tiles
    const int64_t b4 = tiles_bound(p, pl, 4, 4), bL = tiles_bound(p, pl, S0, 3), bS = S0 > 0 ? tiles_bound(p, pl, 0, S0 - 1) : 0;
    auto blocks = [](int64_t work) { return (work + 7) / 8 * 8; };
    // Small tiles two to a 512-thread workgroup in the same launch as the 256-row tiles, or one to a
    // 256-thread workgroup in a launch of their own (then up to three workgroups share a compute unit
    // and run independently; the halves of a pair run in lock step behind one barrier).  Measured: pairs
    // are 3-4 % faster where most rows sit in 256-row tiles and the small tiles are their remainders
    // (fp8 store, 2048 requests x top-8 of 512 chunks) and for light bf16 tiles (about 32 rows per bucket:
    // 256 requests x top-8 of 256 chunks); independent workgroups are 4-8 % faster for bf16 tiles of
    // 64-128 rows (1024 requests x top-16 of 1024 chunks) and up to 35 % faster when the whole launch is
    // only a few workgroups per compute unit or the tiles of an fp8 store carry few rows.
    static const int forced = tuning_env("MOSKA_SHARED_PAIRED", -1);
    const double mean_rows = (double)p.B * p.k * (p.Hq / p.Hkv) / p.C;
    const int64_t items = (int64_t)p.B * p.Hkv * p.k, nb = (int64_t)p.Hkv * p.C;
    const bool many = (items < nb ? items : nb) >= 1024;    // buckets that can be non-empty: >= 4 per compute unit
    int paired = forced >= 0 ? forced
                             : (many && a.nsplit == 1 && (KVD == MOSKA_FP8_E4M3 ? mean_rows >= 128.0 : mean_rows <= 48.0));
    const int64_t grid = blocks(b4) + (paired ? blocks((bL + 1) / 2) + blocks((bS + 1) / 2) : 0);
    int Hq = p.Hq, Hkv = p.Hkv, C = p.C, L = p.L, k = p.k;
    float scale = p.scale;
    SharedArgs args = a;
    void *kargs[] = {&args, &paired, &Hq, &Hkv, &C, &L, &k, &scale};
    const void *kern = a.nsplit > 1 ? (const void *)shared_all_kernel<KVD, 2, true>
                                    : (const void *)shared_all_kernel<KVD, 2, false>;
    if (grid > 0 && hipLaunchKernel(kern, dim3((unsigned)grid, a.nsplit), dim3(512), kargs, 0, s) != hipSuccess)
        return MOSKA_ERR_HIP;
    if (!paired && bL + bS > 0) {
        // an fp8 store's tiles of up to 64 rows have a kernel of their own (three workgroups per compute unit)
        // when there are enough buckets to fill the chip several times; with fewer, two launches one after
        // the other cost more than the third workgroup gains (512 buckets of ~64 rows: 0.20 against 0.15 ms)
        int c_lo = 0;
        int64_t rest = bL + bS;
        if (KVD == MOSKA_FP8_E4M3 && many) {
            const int64_t light = tiles_bound(p, pl, 0, 2);
            void *largs[] = {&args, &Hq, &Hkv, &C, &L, &k, &scale};
            const void *lk = a.nsplit > 1 ? (const void *)shared_light_f8_kernel<2, true>
                                          : (const void *)shared_light_f8_kernel<2, false>;
            if (light > 0 && hipLaunchKernel(lk, dim3((unsigned)blocks(light), a.nsplit), dim3(256), largs, 0, s) != hipSuccess)
                return MOSKA_ERR_HIP;
            c_lo = 3;
            rest = tiles_bound(p, pl, 3, 3);
        }
        void *sargs[] = {&args, &c_lo, &Hq, &Hkv, &C, &L, &k, &scale};
        const void *sk = a.nsplit > 1 ? (const void *)shared_small_kernel<KVD, 2, true>
                                      : (const void *)shared_small_kernel<KVD, 2, false>;
        if (rest > 0 && hipLaunchKernel(sk, dim3((unsigned)blocks(rest), a.nsplit), dim3(256), sargs, 0, s) != hipSuccess)
            return MOSKA_ERR_HIP;
    }
    return MOSKA_OK;
}

}  // namespace mfma
}  // namespace moska
