// Version and error text of libbitsnap.
#include "../../include/bitsnap.h"

extern "C" int bitsnap_version(void) { return 100; /* 0.1.0 */ }

extern "C" const char *bitsnap_error_string(int code)
{
    switch (code) {
    case BITSNAP_OK: return "ok";
    case BITSNAP_E_NULL: return "a required pointer is NULL";
    case BITSNAP_E_SIZE: return "unsupported size, element width, cluster count or group length";
    case BITSNAP_E_ALIGN: return "a pointer is not aligned as required";
    case BITSNAP_E_WORKSPACE: return "workspace missing or too small";
    case BITSNAP_E_OFFSETS: return "tile_offsets requested for a tensor of 2^32 elements or more";
    case BITSNAP_E_LAUNCH: return "the HIP runtime refused the kernel launch";
    default: return "unknown bitsnap error code";
    }
}
