// Prefix-prefill attention (placeholder until the MFMA kernel lands).
#include <hip/hip_runtime.h>

#include "vt_internal.h"

namespace vt {
int launch_prefill(vt_ctx*, const vt_prefill_args*, void*) { return VT_E_UNSUPPORTED; }
}  // namespace vt
