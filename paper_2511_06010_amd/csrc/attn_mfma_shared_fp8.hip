// MFMA Shared KV Attention, fp8-e4m3 shared store (scores on the scaled fp8 MFMA from keys that stay fp8; values
// widened to bf16 for the P V product).
#include "attn_mfma_shared_impl.h"
namespace moska {
int launch_shared_mfma_fp8(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    return mfma::launch_shared_classes<MOSKA_FP8_E4M3>(p, a, pl, s);
}
}  // namespace moska
