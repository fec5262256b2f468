// Launcher of the MFMA Shared KV Attention for one key/value dtype; included by one translation
// unit per dtype so the instantiations compile in parallel.
#pragma once

#include "attn_mfma_lds.h"

namespace moska {
namespace mfma {

// One launch serves every tile (shared_all_kernel): workgroups for the 256-row tiles, for pairs of
// LDS-staged small tiles and, for an fp8 store, for pairs of streaming tiles, each count taken from
// the host-side bound on the tiles of that kind and rounded up to a multiple of 8.
template <int KVD>
int launch_shared_classes(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    constexpr int S0 = KVD == MOSKA_FP8_E4M3 ? 2 : 0;       // first class of the LDS-staged small tiles
    const int64_t b4 = tiles_bound(p, pl, 4, 4), bL = tiles_bound(p, pl, S0, 3), bS = S0 > 0 ? tiles_bound(p, pl, 0, S0 - 1) : 0;
    auto blocks = [](int64_t work) { return (work + 7) / 8 * 8; };
    const int64_t grid = blocks(b4) + blocks((bL + 1) / 2) + blocks((bS + 1) / 2);
    if (grid == 0) return MOSKA_OK;
    int Hq = p.Hq, Hkv = p.Hkv, C = p.C, L = p.L, k = p.k;
    float scale = p.scale;
    SharedArgs args = a;
    void *kargs[] = {&args, &Hq, &Hkv, &C, &L, &k, &scale};
    const void *kern = a.nsplit > 1 ? (const void *)shared_all_kernel<KVD, 2, true>
                                    : (const void *)shared_all_kernel<KVD, 2, false>;
    if (hipLaunchKernel(kern, dim3((unsigned)grid, a.nsplit), dim3(512), kargs, 0, s) != hipSuccess) return MOSKA_ERR_HIP;
    return MOSKA_OK;
}

}  // namespace mfma
}  // namespace moska
