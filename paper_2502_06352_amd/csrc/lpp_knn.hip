#include "lpp_internal.h"
extern "C" size_t lpp_build_neighbours_workspace(int32_t, int32_t, int32_t) { return 256; }
extern "C" int32_t lpp_build_neighbours(const float*, int32_t, int32_t, int32_t, int32_t*, void*, size_t, void*) {
  return LPP_EUNSUPPORTED;
}
