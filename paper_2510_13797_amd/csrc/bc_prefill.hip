// bc_prefill_attn: beacon-masked prefill attention (Fig. 2, Sec. 3.2).  Placeholder until the
// MFMA kernel lands: reports the shape as unsupported instead of computing anything.
#include "bc_common.h"

extern "C" int32_t bc_prefill_attn(const bc_shape*, const void*, const void*, const void*,
                                   const int64_t*, const int32_t*, const int32_t*, int32_t, float*,
                                   float*, void*) {
  return BC_ERR_SHAPE;
}
