// MFMA Unique KV Attention launcher and the dispatch of the MFMA Shared KV Attention variants.
#include <cstdlib>

#include "attn_mfma.h"

namespace moska {

int launch_shared_mfma_bf16(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s);
int launch_shared_mfma_fp8(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s);

int launch_shared_mfma(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    return p.shared_kv_dtype == MOSKA_FP8_E4M3 ? launch_shared_mfma_fp8(p, a, pl, s)
                                               : launch_shared_mfma_bf16(p, a, pl, s);
}

int launch_unique_mfma(const moska_problem_t &p, const UniqueArgs &a, hipStream_t s) {
    using namespace mfma;
    struct UniqueVariant {
        Variant v;
        const void *kernel;
    };
#define MOSKA_UV(NR, NW, AUX, NKB) \
    UniqueVariant { Variant{NR, NW, AUX, NKB}, (const void *)unique_mfma_kernel<NR, NW, AUX, NKB> }
    // first entry of each row count is the default; MOSKA_UNIQUE_VARIANT=<index> picks another
    static const UniqueVariant table[] = {
        MOSKA_UV(1, 4, 2, 1), MOSKA_UV(1, 4, 2, 2), MOSKA_UV(1, 8, 2, 1), MOSKA_UV(2, 4, 2, 1), MOSKA_UV(4, 4, 2, 2),
    };
#undef MOSKA_UV
    const int G = p.Hq / p.Hkv;
    const int NR = G <= 16 ? 1 : G <= 32 ? 2 : 4;
    int want = 0;
    if (const char *e = std::getenv("MOSKA_UNIQUE_VARIANT")) want = std::atoi(e);
    const UniqueVariant *pick = nullptr;
    int seen = 0;
    for (const UniqueVariant &uv : table)
        if (uv.v.NR == NR) {
            if (!pick || seen == want) pick = &uv;
            ++seen;
        }
    const int gt = (G + 16 * NR - 1) / (16 * NR);
    const unsigned grid = (unsigned)((int64_t)p.B * p.Hkv * gt);
    UniqueArgs args = a;
    int Hq = p.Hq, Hkv = p.Hkv, U = p.U_max, k = p.k;
    float scale = p.scale;
    void *kargs[] = {&args, &Hq, &Hkv, &U, &k, &scale};
    return hip_status(hipLaunchKernel(pick->kernel, dim3(grid), dim3(pick->v.NW * 64), kargs, 0, s));
}

}  // namespace moska
