// Error-code descriptions of the C ABI.
#include "cwac.h"

extern "C" const char *cwac_status_string(cwac_status s) {
  switch (s) {
    case CWAC_OK: return "ok";
    case CWAC_E_NULL: return "a required pointer is NULL";
    case CWAC_E_SHAPE: return "a size is out of the supported range";
    case CWAC_E_ALIGN: return "a pointer or leading dimension violates the required alignment";
    case CWAC_E_MODE: return "inconsistent mode or optional-argument combination";
    case CWAC_E_WORKSPACE: return "workspace missing or too small";
    case CWAC_E_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
  }
}
