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

// One launch per tile size class of the plan.  Small tiles (16, 32 rows) go to the streaming
// kernels, whose registers hold every row; tiles of 64 rows and more go to the LDS-staged
// kernels, where the waves split the rows and share each K/V stage.
template <int KVD>
int launch_shared_classes(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    static const SharedKernel table[] = {
        {0, 256, (const void *)shared_mfma_kernel<1, KVD, 4, 2, 1>},
        {1, 256, (const void *)shared_mfma_kernel<2, KVD, 4, 2, 1>},
        {2, 256, (const void *)shared_lds_kernel<1, 4, KVD, 2, MIXED_KT, 1>},   // as in the mixed launch
        {3, 256, (const void *)shared_lds_kernel<2, 4, KVD, 2, MIXED_KT, 1>},
        {4, 512, (const void *)shared_lds_kernel<2, 8, KVD, 2, 64, 2>},
    };
    // tuning overrides: MOSKA_SHARED_C64=stream serves 64-row tiles with the streaming kernel;
    // MOSKA_SHARED_MIXED=0 launches every class on its own instead of classes 0..3 together
    static const SharedKernel c64_stream = {2, 256, (const void *)shared_mfma_kernel<4, KVD, 4, 2, 1>};
    static const bool use_c64_stream = [] {
        const char *e = std::getenv("MOSKA_SHARED_C64");
        return e && e[0] == 's';
    }();
    static const bool mixed = [] {
        const char *e = std::getenv("MOSKA_SHARED_MIXED");
        return !(e && e[0] == '0');
    }();
    static const int small = [] {
        const char *e = std::getenv("MOSKA_SHARED_SMALL");
        return e ? std::atoi(e) : 0;
    }();
    static const void *small_kernels[] = {
        nullptr,
        (const void *)shared_small_kernel<KVD, 2, 64, 1, 2>,
        (const void *)shared_small_kernel<KVD, 2, 32, 1, 3>,
        (const void *)shared_small_kernel<KVD, 2, 32, 2, 3>,
        (const void *)shared_small_kernel<KVD, 2, 64, 2, 2>,
        (const void *)shared_small_kernel<KVD, 2, 32, 1, 4>,
    };
    int Hq = p.Hq, Hkv = p.Hkv, C = p.C, L = p.L, k = p.k;
    float scale = p.scale;
    SharedArgs args = a;
    int top = pl.cmin - 1;                                      // classes <= top go to the mixed launch
    if (mixed && !use_c64_stream) top = pl.cmax < 3 ? pl.cmax : 3;
    if (small > 0 && small < 6) top = pl.cmax < 2 ? pl.cmax : 2;
    for (int c = pl.cmax; c >= pl.cmin && c > top; --c) {      // big tiles first: they run longest
        const int64_t bound = class_bound(p, pl, c);
        if (bound == 0) continue;
        const SharedKernel &sk = (c == 2 && use_c64_stream) ? c64_stream : table[c];
        const unsigned grid = (unsigned)(((bound + 7) / 8) * 8);
        int cls = c;
        void *kargs[] = {&args, &cls, &Hq, &Hkv, &C, &L, &k, &scale};
        if (hipLaunchKernel(sk.kernel, dim3(grid, a.nsplit), dim3(sk.threads), kargs, 0, s) != hipSuccess) return MOSKA_ERR_HIP;
    }
    if (small > 0 && small < 6) {
        int c0 = pl.cmin, c1 = pl.cmax < 2 ? pl.cmax : 2;
        int64_t bound = 0;
        for (int c = c0; c <= c1; ++c) bound += class_bound(p, pl, c);
        if (c0 <= c1 && bound > 0) {
            const unsigned grid = (unsigned)(((bound + 7) / 8) * 8);
            void *kargs[] = {&args, &c0, &c1, &Hq, &Hkv, &C, &L, &k, &scale};
            if (hipLaunchKernel(small_kernels[small], dim3(grid, a.nsplit), dim3(256), kargs, 0, s) != hipSuccess)
                return MOSKA_ERR_HIP;
        }
    } else if (mixed && !use_c64_stream) {
        int c0 = pl.cmin, c1 = pl.cmax < 3 ? pl.cmax : 3;
        int64_t bound = 0;
        for (int c = c0; c <= c1; ++c) bound += class_bound(p, pl, c);
        if (c0 <= c1 && bound > 0) {
            const unsigned grid = (unsigned)(((bound + 7) / 8) * 8);
            void *kargs[] = {&args, &c0, &c1, &Hq, &Hkv, &C, &L, &k, &scale};
            static const bool pd2 = [] {
                const char *e = std::getenv("MOSKA_SHARED_PD1");
                return e && e[0] == '2';
            }();
            const void *mk = pd2 ? (const void *)shared_mixed_kernel<KVD, 2, 2> : (const void *)shared_mixed_kernel<KVD, 2, 1>;
            if (hipLaunchKernel(mk, dim3(grid, a.nsplit), dim3(256), kargs, 0, s) != hipSuccess)
                return MOSKA_ERR_HIP;
        }
    }
    return MOSKA_OK;
}

}  // namespace mfma
}  // namespace moska
