// Dense (prefill, batch >= 64) path -- placeholder until the MFMA GEMM kernels land.
#include "nq_internal.h"

namespace nq {

size_t prefill_workspace_bytes(int64_t, int64_t, int64_t, int) { return 0; }

int launch_prefill(const PrefillArgs&, hipStream_t)
{
    set_error("prefill path not built");
    return NQ_E_UNSUPPORTED;
}

}  // namespace nq
