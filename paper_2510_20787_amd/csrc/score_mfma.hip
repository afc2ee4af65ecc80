// placeholder until the MFMA scoring kernel lands
#include "ltea_common.h"
#include "ltea_kernels.h"
namespace ltea {
bool score_mfma_supported(const ltea_cfg&, const ltea_cnn&) { return false; }
hipError_t launch_score_mfma(const ltea_cfg&, const ltea_cnn&, const void*, const void*, int64_t, int64_t,
                             const SeqView&, float*, hipStream_t) { return hipErrorNotSupported; }
}
