// MFMA Shared KV Attention, bf16 shared store.
#include "attn_mfma_shared_impl.h"
namespace moska {
int launch_shared_mfma_bf16(const moska_problem_t &p, const SharedArgs &a, const SharedPlan &pl, hipStream_t s) {
    return mfma::launch_shared_classes<MOSKA_BF16>(p, a, pl, s);
}
}  // namespace moska
