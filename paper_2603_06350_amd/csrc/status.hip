// moe_strerror: text for the status codes of include/moe.h.
#include "moe_internal.h"

extern "C" const char* moe_strerror(int code) {
  switch (code) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument (null or misaligned pointer, or bad shape)";
    case MOE_ERR_UNSUPPORTED: return "shape outside the supported limits";
    case MOE_ERR_WORKSPACE: return "workspace too small";
    case MOE_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}
