// The format-dependent kernels and their launch logic for the BF16 cache format, head_dim 128.
#include "ts_fused.h"

namespace ts {
TS_FORMAT_FUNCTIONS(, TS_KV_BF16, 128)
}  // namespace ts
