// Entry points that are not tied to one kernel file.
#include "gr_internal.hpp"

extern "C" const char* gr_status_string(gr_status s) {
  switch (s) {
    case GR_OK: return "GR_OK";
    case GR_ERR_INVALID_ARG: return "GR_ERR_INVALID_ARG: null pointer, bad size, step or u out of range, or aliasing rule broken";
    case GR_ERR_UNSUPPORTED: return "GR_ERR_UNSUPPORTED: shape outside what the gfx950 kernels implement";
    case GR_ERR_WORKSPACE_TOO_SMALL: return "GR_ERR_WORKSPACE_TOO_SMALL";
    case GR_ERR_BAD_TABLE: return "GR_ERR_BAD_TABLE: item table unsorted, has duplicates, or a token outside [0, V)";
    case GR_ERR_HIP: return "GR_ERR_HIP: HIP runtime call or kernel launch failed";
    default: return "unknown gr_status";
  }
}
