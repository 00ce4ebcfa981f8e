// The format-dependent kernels and their launch logic for the INT8 cache format, head_dim 128.
#include "ts_fused.h"

namespace ts {
TS_FORMAT_FUNCTIONS(, TS_KV_INT8, 128)
}  // namespace ts
