// Status strings and ABI version of the dynamic-bottleneck library.
#include "laud_common.h"

extern "C" const char* laud_status_string(int status) {
  switch (status) {
    case LAUD_OK: return "LAUD_OK";
    case LAUD_ERR_INVALID_ARG: return "LAUD_ERR_INVALID_ARG: null pointer, bad dimension, or S/D does not divide";
    case LAUD_ERR_UNSUPPORTED: return "LAUD_ERR_UNSUPPORTED: dtype or shape outside what the kernels cover";
    case LAUD_ERR_WORKSPACE: return "LAUD_ERR_WORKSPACE: workspace missing or too small";
    case LAUD_ERR_HIP: return "LAUD_ERR_HIP: kernel launch failed";
    default: return "LAUD: unknown status";
  }
}

extern "C" int laud_abi_version(void) { return 1; }
