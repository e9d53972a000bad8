// bf16 MFMA kernel family for p = 2 (placeholder: not built yet, every problem is unsupported).
#include "common.hpp"

namespace pa {
pa_status mfma_supported(const pa_problem&) { return PA_ERR_UNSUPPORTED; }
size_t mfma_workspace_bytes(const pa_problem&, bool) { return 0; }
long long mfma_state_rows(const pa_problem&) { return 0; }
pa_status mfma_fwd(const Ctx&, const void*, const void*, const void*, void*, float*) { return PA_ERR_UNSUPPORTED; }
pa_status mfma_bwd(const Ctx&, const void*, const void*, const void*, const void*, const float*, const void*, void*,
                   void*, void*) {
    return PA_ERR_UNSUPPORTED;
}
}  // namespace pa
