// Status strings and version of libjz.
#include "jz_internal.h"

extern "C" const char* jz_status_string(int status) {
  switch (status) {
    case JZ_OK: return "JZ_OK";
    case JZ_ERR_NULL: return "JZ_ERR_NULL: a required pointer is NULL";
    case JZ_ERR_SHAPE: return "JZ_ERR_SHAPE: invalid dimensions or table";
    case JZ_ERR_UNSUPPORTED: return "JZ_ERR_UNSUPPORTED: valid request that this build does not implement";
    case JZ_ERR_WORKSPACE: return "JZ_ERR_WORKSPACE: workspace missing or too small";
    case JZ_ERR_ALIGN: return "JZ_ERR_ALIGN: device pointer not 16-byte aligned";
    case JZ_ERR_ALIAS: return "JZ_ERR_ALIAS: output overlaps an input or the workspace";
    case JZ_ERR_LAUNCH: return "JZ_ERR_LAUNCH: HIP runtime error at launch";
    case JZ_ERR_NOT_PREPARED: return "JZ_ERR_NOT_PREPARED: LARS workspace not prepared for this parameter set";
    default: return "unknown libjz status";
  }
}

extern "C" int jz_version(void) { return 110; }
