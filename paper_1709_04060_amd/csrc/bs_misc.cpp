// Status strings and version of libbsgemm.
#include "bsgemm.h"

extern "C" const char *bs_status_string(bs_status s)
{
    switch (s) {
    case BS_OK: return "ok";
    case BS_ERR_INVALID_ARG: return "invalid argument";
    case BS_ERR_UNSUPPORTED: return "unsupported configuration";
    case BS_ERR_ALIGNMENT: return "misaligned pointer or leading dimension";
    case BS_ERR_OVERFLOW_RISK: return "int32 accumulator or 32-bit index could overflow";
    case BS_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

extern "C" int bs_version(void) { return 100; }
