// Kernel table and launcher of the MFMA Shared KV Attention for one key/value dtype; included by
// one translation unit per dtype so the instantiations compile in parallel.
#pragma once

#include <cstdlib>

#include "attn_mfma_lds.h"

namespace moska {
namespace mfma {

struct SharedKernel {
    int cls;            // tile size class served
    int threads;
    const void *kernel;
};

// Tiles of up to 128 rows go out in one launch (shared_mixed_kernel), the 256-row class in a launch
// of its own, issued first because its tiles run longest.  MOSKA_SHARED_MIXED=0 (tuning) launches
// every class on its own instead.
template <int KVD>
int launch_shared_classes(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    // [split run?][class]: the slices of a split run are written for the combine kernel (write-back), whole
    // results with the non-temporal hint
    static const SharedKernel table[2][5] = {
        {{0, 256, (const void *)shared_mfma_kernel<1, KVD, 4, 2, 1, false>},
         {1, 256, (const void *)shared_mfma_kernel<2, KVD, 4, 2, 1, false>},
         {2, 256, (const void *)shared_lds_kernel<1, 4, KVD, 2, MIXED_KT, 1, false>},   // as in the mixed launch
         {3, 256, (const void *)shared_lds_kernel<2, 4, KVD, 2, MIXED_KT, 1, false>},
         {4, 512, (const void *)shared_lds_kernel<2, 8, KVD, 2, 64, 2, false>}},
        {{0, 256, (const void *)shared_mfma_kernel<1, KVD, 4, 2, 1, true>},
         {1, 256, (const void *)shared_mfma_kernel<2, KVD, 4, 2, 1, true>},
         {2, 256, (const void *)shared_lds_kernel<1, 4, KVD, 2, MIXED_KT, 1, true>},
         {3, 256, (const void *)shared_lds_kernel<2, 4, KVD, 2, MIXED_KT, 1, true>},
         {4, 512, (const void *)shared_lds_kernel<2, 8, KVD, 2, 64, 2, true>}},
    };
    const bool split = a.nsplit > 1;
    static const bool mixed = [] {
        const char *e = std::getenv("MOSKA_SHARED_MIXED");
        return !(e && e[0] == '0');
    }();
    int Hq = p.Hq, Hkv = p.Hkv, C = p.C, L = p.L, k = p.k;
    float scale = p.scale;
    SharedArgs args = a;
    const int top = !mixed ? pl.cmin - 1 : pl.cmax < 3 ? pl.cmax : 3;   // classes <= top go to the mixed launch
    for (int c = pl.cmax; c >= pl.cmin && c > top; --c) {
        const int64_t bound = class_bound(p, pl, c);
        if (bound == 0) continue;
        const SharedKernel &sk = table[split][c];
        const unsigned grid = (unsigned)(((bound + 7) / 8) * 8);
        int cls = c;
        void *kargs[] = {&args, &cls, &Hq, &Hkv, &C, &L, &k, &scale};
        if (hipLaunchKernel(sk.kernel, dim3(grid, a.nsplit), dim3(sk.threads), kargs, 0, s) != hipSuccess) return MOSKA_ERR_HIP;
    }
    if (mixed) {
        int c0 = pl.cmin, c1 = top;
        int64_t bound = 0;
        for (int c = c0; c <= c1; ++c) bound += class_bound(p, pl, c);
        if (c0 <= c1 && bound > 0) {
            const unsigned grid = (unsigned)(((bound + 7) / 8) * 8);
            void *kargs[] = {&args, &c0, &c1, &Hq, &Hkv, &C, &L, &k, &scale};
            const void *mk = split ? (const void *)shared_mixed_kernel<KVD, 2, true>
                                   : (const void *)shared_mixed_kernel<KVD, 2, false>;
            if (hipLaunchKernel(mk, dim3(grid, a.nsplit), dim3(256), kargs, 0, s) != hipSuccess)
                return MOSKA_ERR_HIP;
        }
    }
    return MOSKA_OK;
}

}  // namespace mfma
}  // namespace moska
