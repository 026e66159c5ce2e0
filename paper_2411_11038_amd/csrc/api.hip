// Library-level entry points that are not tied to one kernel family.
#include "common.hpp"

extern "C" int efqat_version(void) { return EFQAT_VERSION; }

extern "C" const char* efqat_strerror(int code) {
  switch (code) {
    case EFQAT_OK: return "ok";
    case EFQAT_ERR_NULL_PTR: return "a required pointer is NULL";
    case EFQAT_ERR_BAD_SHAPE: return "a dimension is non-positive or too large";
    case EFQAT_ERR_BAD_BITS: return "bit width outside 2..8";
    case EFQAT_ERR_BAD_K: return "k outside 0..C_out";
    case EFQAT_ERR_BAD_LAYOUT: return "unknown layout / mode flag";
    case EFQAT_ERR_WORKSPACE: return "workspace too small";
    case EFQAT_ERR_HIP: return "a HIP call or kernel launch failed";
    case EFQAT_ERR_BAD_DTYPE: return "unknown element type";
    case EFQAT_ERR_ALIGNMENT: return "a pointer is not aligned as required";
    default: return "unknown error code";
  }
}
