// bf16 variant of the dense layer update (bf16 MFMA, fp32 accumulate).
#include "common.h"

fg_status_t fg_launch_linear_bf16(const void*, int32_t, int64_t, fg_dtype_t, const void*, int64_t, const int32_t*,
                                  const int64_t*, int64_t, int32_t, int32_t, const void*, const float*, int32_t, void*,
                                  int32_t, int64_t, fg_dtype_t, hipStream_t) {
    FG_FAIL(FG_ERR_DTYPE, "fg_linear: the bf16 path is not built yet");
}
