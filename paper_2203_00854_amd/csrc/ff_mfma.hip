// bf16 matrix-core kernel family (placeholder while the generic family is validated).
#include "ff_common.h"

namespace ff {
bool mfma_supported(const Problem&) { return false; }
size_t mfma_workspace(const Problem&, int, Workspace*, void*) { return 0; }
ff_status mfma_bias(const Problem&, const ff_attn_weights&, const void*, const void*, const Workspace&, hipStream_t) {
    return fail(FF_EUNSUPPORTED, "matrix-core family not built");
}
ff_status mfma_chunk(const Problem&, const ff_attn_weights&, const void*, const float*, void*, const Workspace&, int,
                     int, hipStream_t) {
    return fail(FF_EUNSUPPORTED, "matrix-core family not built");
}
}  // namespace ff
