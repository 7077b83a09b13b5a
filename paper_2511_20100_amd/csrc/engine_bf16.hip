// bf16 path schedulers (weights and KV cache in bf16, fp32 residual stream and accumulators).
#include "engine.h"
#include "kernels.h"

namespace mtmc {

void bf16_plan_rollout_extra(const mtmc_weights*, RolloutPlan&, Carver&) {}
void bf16_plan_score_extra(const mtmc_weights*, ScorePlan&, Carver&) {}

int bf16_store_weights(mtmc_weights*, const BlobLayout&, const void*, bool, hipStream_t) {
  set_error("MTMC_BF16 is not available in this build");
  return MTMC_EINVAL;
}
int bf16_rollout(const mtmc_weights*, const RolloutPlan&, const int*, const SampleArgs&, hipStream_t) {
  set_error("MTMC_BF16 is not available in this build");
  return MTMC_EINVAL;
}
int bf16_score(const mtmc_weights*, const ScorePlan&, const ScoreArgs&, hipStream_t) {
  set_error("MTMC_BF16 is not available in this build");
  return MTMC_EINVAL;
}

}  // namespace mtmc
