// bf16 MFMA scoring path (placeholder until the kernels land: nothing is routed here).
#include "common.h"

namespace adakv {

bool mfma_path_supported(const Dims &, int) { return false; }

hipError_t launch_score_mfma(const SeqTab &, const Dims &, const void *, const void *,
                             const float *, float *, char *, const ScorePlan &, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace adakv
