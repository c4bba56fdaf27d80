#include "lpp_internal.h"
extern "C" size_t lpp_tree_attention_workspace(const lpp_tree*, int32_t, int32_t, int32_t, int32_t) { return 256; }
extern "C" int32_t lpp_tree_attention(const lpp_tree*, int32_t, const void*, const void*, const void*, const void*,
                                      const void*, const int32_t*, int32_t, int32_t, int32_t, int32_t, float,
                                      float*, void*, size_t, void*) { return LPP_EUNSUPPORTED; }
