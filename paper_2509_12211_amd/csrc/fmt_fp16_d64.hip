// The format-dependent kernels and their launch logic for the FP16 cache format, head_dim 64.
#include "ts_fused.h"

namespace ts {
TS_FORMAT_FUNCTIONS(, TS_KV_FP16, 64)
}  // namespace ts
