// Matrix-core (MFMA) kernel family for bf16 tensors.
#include "bra_common.h"

namespace bra {

bool mfma_supported(const Dims &) { return false; }
size_t mfma_workspace_bytes(const Dims &) { return 0; }
int mfma_route(const Dims &, const void *, const void *, int32_t *, float *, void *, hipStream_t)
{
    return BRA_ERR_UNSUPPORTED;
}
int mfma_forward(const Dims &, const void *, const void *, const void *, const void *, void *,
                 int32_t *, const int32_t *, void *, hipStream_t)
{
    return BRA_ERR_UNSUPPORTED;
}

}  // namespace bra
