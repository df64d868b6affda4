// Backward reduce kernels with the SGD row update.
#include "bwd_reduce.h"

namespace dlrm {
int run_reduce_sgd(const GroupArgs& g, const UpdArgs& u, int dtype, int G, int K,
    const dlrm_bwd_timing* tm, hipStream_t st) {
  return run_reduce<kSgd, false>(g, u, dtype, G, K, tm, st);
}
}  // namespace dlrm
