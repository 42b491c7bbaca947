// MFMA path (placeholder while the tiles are being written): reports itself
// unavailable, so the scheduler never selects it.
#include "dfk_internal.h"

namespace dfk {
bool mfma_config_valid(const dfk_config_t&, int, int, int, dfk_dtype_t) { return false; }
int mfma_max_tokens_per_launch() { return 64; }
hipError_t launch_mfma(const MlpArgs&, const dfk_config_t&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace dfk
