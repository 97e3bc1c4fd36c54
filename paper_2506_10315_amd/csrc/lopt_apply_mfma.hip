// Matrix-core variant of the fused apply pass (hidden width 32). Placeholder until the
// MFMA kernel lands: reports itself unavailable so the vector-ALU kernel is used.
#include "lopt_internal.h"

namespace lopt {

bool apply_mfma_available(const StepArgs&) { return false; }
void launch_apply_mfma(const Launch&, const StepArgs&, const WeightsDev&, hipStream_t) {}

}  // namespace lopt
