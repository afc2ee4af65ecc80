// placeholder until the MFMA attention kernel lands
#include "ltea_common.h"
#include "ltea_kernels.h"
namespace ltea {
bool attention_mfma_supported(const ltea_cfg&) { return false; }
hipError_t launch_attention_mfma(const ltea_cfg&, const void*, int64_t, int64_t, const void*, const void*, int64_t,
                                 int64_t, const SeqView&, const ltea_cache&, void*, hipStream_t) { return hipErrorNotSupported; }
}
