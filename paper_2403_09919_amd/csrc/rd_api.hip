// Status strings and version of the rd library.
#include "rd_internal.h"

extern "C" const char *rd_strerror(int code)
{
    switch (code) {
    case RD_OK: return "ok";
    case RD_ERR_INVALID_ARG: return "invalid argument (null pointer, non-positive size or misaligned buffer)";
    case RD_ERR_UNSUPPORTED: return "unsupported size or dtype (limits: W <= 128, W*L <= 384, D in {64,128})";
    case RD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case RD_ERR_HIP: return "HIP kernel launch failed";
    default: return "unknown rd status";
    }
}

extern "C" int rd_version(void) { return 100; }
