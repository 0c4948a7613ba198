// Causal attention on the matrix cores (placeholder until the MFMA kernel lands: reports that
// no shape is supported, so the plain kernel serves every call).
#include "zo_kernels.h"

namespace zo {

bool mfma_attention_supported(int, int) { return false; }

hipError_t launch_attention_mfma(const void *, void *, int, int, int, int, int, hipStream_t)
{
    return hipErrorNotSupported;
}

}  // namespace zo
