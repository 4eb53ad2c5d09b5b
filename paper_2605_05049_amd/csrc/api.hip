// Host-only entry points of the C ABI: status strings, workspace size, version.
#include "common.h"

extern "C" const char* moe_status_str(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_NULL: return "a required pointer is NULL";
    case MOE_ERR_SHAPE: return "shape outside the supported limits";
    case MOE_ERR_ALIGN: return "pointer not sufficiently aligned";
    case MOE_ERR_WORKSPACE: return "workspace too small";
    case MOE_ERR_RUNTIME: return "HIP launch failed";
    default: return "unknown status";
  }
}

extern "C" size_t moe_workspace_bytes(const moe_shape* shape) {
  moe::Dims D;
  if (moe::check_shape(shape, &D) != MOE_OK) return 0;
  return moe::ws_layout(D).total;
}

extern "C" int moe_abi_version(void) { return 1; }
