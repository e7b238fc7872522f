// MFMA kernel family: dispatch table (kernels are added per shape family).
#include "monarch_internal.h"

namespace monarch {

bool mfma_fwd_supported(const Problem&) { return false; }
bool mfma_bwd_supported(const Problem&) { return false; }
size_t mfma_bwd_workspace(const Problem&) { return 0; }
const char* mfma_fwd_name(const Problem&) { return "unsupported"; }
const char* mfma_bwd_name(const Problem&) { return "unsupported"; }
int mfma_fwd(const Problem&, const void*, const void*, const void*, void*, hipStream_t) { return -2; }
int mfma_bwd(const Problem&, const void*, const void*, const void*, const void*, void*, void*, void*, void*,
             hipStream_t)
{
    return -2;
}

}  // namespace monarch
