// Status strings of the LowDiff C ABI.
#include "ld_common.h"

extern "C" const char* ld_status_string(ld_status s) {
    switch (s) {
        case LD_OK: return "LD_OK";
        case LD_ERR_NULL: return "LD_ERR_NULL: a required pointer is NULL";
        case LD_ERR_RANGE: return "LD_ERR_RANGE: a size, count or table entry is out of range";
        case LD_ERR_WORKSPACE: return "LD_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case LD_ERR_HIP: return "LD_ERR_HIP: a HIP runtime call or kernel launch failed";
        case LD_ERR_ALIGN: return "LD_ERR_ALIGN: a device pointer is not aligned as required";
        default: return "unknown ld_status";
    }
}
