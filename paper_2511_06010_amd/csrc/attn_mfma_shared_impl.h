// Variant table and launcher of the MFMA Shared KV Attention kernel for one key/value dtype;
// included by one translation unit per dtype so the instantiations compile in parallel.
#pragma once

#include <cstdlib>

#include "attn_mfma.h"

namespace moska {
namespace mfma {

struct SharedVariant {
    Variant v;
    const void *kernel;
};

template <int KVD>
int launch_shared_variant(const moska_problem_t &p, const SharedArgs &a, int MT, hipStream_t s) {
#define MOSKA_SV(NR, NW, AUX, NKB) \
    SharedVariant { Variant{NR, NW, AUX, NKB}, (const void *)shared_mfma_kernel<NR, KVD, NW, AUX, NKB> }
    // first entry of each row count is the default; the others are reachable through
    // MOSKA_SHARED_VARIANT=<index within that row count> for tuning runs
    static const SharedVariant table[] = {
        MOSKA_SV(1, 4, 0, 1), MOSKA_SV(1, 4, 2, 1), MOSKA_SV(2, 4, 0, 1), MOSKA_SV(2, 4, 2, 1), MOSKA_SV(2, 4, 2, 2),
        MOSKA_SV(4, 4, 2, 2), MOSKA_SV(4, 4, 2, 1), MOSKA_SV(4, 4, 0, 2),
    };
#undef MOSKA_SV
    const int NR = MT / 16;
    int want = 0;
    if (const char *e = std::getenv("MOSKA_SHARED_VARIANT")) want = std::atoi(e);
    const SharedVariant *pick = nullptr;
    int seen = 0;
    for (const SharedVariant &sv : table)
        if (sv.v.NR == NR) {
            if (!pick || seen == want) pick = &sv;
            ++seen;
        }
    if (!pick || MT % 16) return MOSKA_ERR_UNSUPPORTED;
    const int64_t tmax = max_tiles(p, MT);
    if (tmax == 0) return MOSKA_OK;
    const unsigned grid = (unsigned)(((tmax + 7) / 8) * 8);
    SharedArgs args = a;
    int Hq = p.Hq, Hkv = p.Hkv, C = p.C, L = p.L, k = p.k;
    float scale = p.scale;
    void *kargs[] = {&args, &Hq, &Hkv, &C, &L, &k, &scale};
    return hip_status(hipLaunchKernel(pick->kernel, dim3(grid), dim3(pick->v.NW * 64), kargs, 0, s));
}

}  // namespace mfma
}  // namespace moska
