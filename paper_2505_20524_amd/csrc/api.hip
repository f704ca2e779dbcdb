// Status strings and version of the C ABI.
#include "launch.h"

extern "C" const char* fog_status_string(fog_status s) {
  switch (s) {
    case FOG_OK: return "ok";
    case FOG_ERR_NULL: return "a required pointer is NULL";
    case FOG_ERR_SHAPE: return "bad size or leading dimension";
    case FOG_ERR_ALIGN: return "pointer or leading dimension misaligned";
    case FOG_ERR_UNSUPPORTED: return "problem not covered by the kernels";
    case FOG_ERR_WORKSPACE: return "workspace missing or too small";
    case FOG_ERR_HIP: return "HIP runtime error at launch";
  }
  return "unknown status";
}

extern "C" int fog_version(void) { return 100; }
