// The format-dependent kernels and their launch logic for the FP16 cache format.
#include "ts_fused.h"

namespace ts {
TS_FORMAT_FUNCTIONS(, TS_KV_FP16)
}  // namespace ts
