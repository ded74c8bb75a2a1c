// Status strings, version and per-thread device error of libsdvg.
#include "sdvg_common.h"

namespace sdvg {
thread_local int g_last_device_error = 0;
}

extern "C" const char *sdvg_status_string(int status) {
  switch (status) {
    case SDVG_OK: return "SDVG_OK";
    case SDVG_ERR_NULL: return "SDVG_ERR_NULL: required pointer is NULL";
    case SDVG_ERR_SHAPE: return "SDVG_ERR_SHAPE: non-positive or inconsistent size";
    case SDVG_ERR_RANGE: return "SDVG_ERR_RANGE: slot, length or threshold out of range";
    case SDVG_ERR_ALIGN: return "SDVG_ERR_ALIGN: pointer not 16-byte aligned or stride not a multiple of 8";
    case SDVG_ERR_UNSUPPORTED: return "SDVG_ERR_UNSUPPORTED: head_dim != 128, unknown dtype or mode";
    case SDVG_ERR_DEVICE: return "SDVG_ERR_DEVICE: HIP runtime call failed";
    default: return status > 0 ? "SDVG positive result" : "SDVG unknown status";
  }
}

extern "C" int sdvg_last_device_error(void) { return sdvg::g_last_device_error; }

extern "C" int sdvg_version(void) { return 100; }
