// The format-dependent kernels and their launch logic for the BF16 cache format.
#include "ts_fused.h"

namespace ts {
TS_FORMAT_FUNCTIONS(, TS_KV_BF16)
}  // namespace ts
