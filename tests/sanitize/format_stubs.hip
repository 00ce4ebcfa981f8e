// Stand-ins for the per-format kernel files of the library, for the sanitizer run of its
// entry-point file alone: nothing in that run gets as far as a launch.
#include "ts_fused.h"

namespace ts {
#define TS_STUB(FMT, DD)                                                                        \
  template <>                                                                                   \
  int launch_fused_format<FMT, DD>(const ts_layout*, FusedParams&, const Plan&, const void*,    \
                                   const void*, int, void*) { return TS_ERR_UNSUPPORTED; }      \
  template <>                                                                                   \
  int launch_attention_format<FMT, DD>(const ts_layout*, const AttendParams&, const Plan&,      \
                                       const int32_t*, const int32_t*, int32_t*, void*) {       \
    return TS_ERR_UNSUPPORTED;                                                                  \
  }                                                                                             \
  template <>                                                                                   \
  int append_capacity_format<FMT, DD>(const ts_layout*, const Plan&) { return 0; }
TS_STUB(TS_KV_BF16, 64)
TS_STUB(TS_KV_BF16, 128)
TS_STUB(TS_KV_FP16, 64)
TS_STUB(TS_KV_FP16, 128)
TS_STUB(TS_KV_INT8, 64)
TS_STUB(TS_KV_INT8, 128)
}  // namespace ts
