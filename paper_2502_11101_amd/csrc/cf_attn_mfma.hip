// 16-bit MFMA prefill attention (placeholder until the kernel lands: nothing routes here yet).
#include "cf_common.h"

namespace cf {

bool mfma_path_supported(const cf_layer_desc*) { return false; }
size_t mfma_workspace_bytes(const cf_layer_desc*, int32_t, int32_t, int32_t, int64_t) { return 0; }
cf_status launch_attention_mfma(const AttnArgs&, const RopeFreq&, hipStream_t) {
    set_error("MFMA path not built");
    return CF_ERR_UNSUPPORTED;
}

}  // namespace cf
