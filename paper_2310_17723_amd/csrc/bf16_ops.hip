// BF16 side of a switched module (paper Sec. 2.3, Table 1): placeholder entry points.
#include "hero_common.h"

extern "C" hero_status hero_bf16_gemm(const void*, int64_t, const void*, int64_t, const float*, const void*, int64_t,
                                      int, void*, int64_t, int64_t, int64_t, int64_t, void*) {
    return HERO_ERR_UNSUPPORTED;
}
extern "C" hero_status hero_bf16_attn(const void*, const int64_t*, const void*, const int64_t*, const void*,
                                      const int64_t*, int64_t, int64_t, int64_t, int64_t, int64_t, float, hero_mask,
                                      const int32_t*, void*, int64_t, void*) {
    return HERO_ERR_UNSUPPORTED;
}
