// Status strings and version of the C ABI.
#include "grass_device.h"

extern "C" const char* grass_strerror(int status) {
    switch (status) {
        case GRASS_OK: return "ok";
        case GRASS_EINVAL: return "invalid argument";
        case GRASS_EWORKSPACE: return "workspace missing, misaligned or too small";
        case GRASS_EHIP: return "HIP runtime error";
        case GRASS_EUNSUPPORTED: return "request outside the supported range";
        case GRASS_ETOOLARGE: return "problem needs more scratch memory than the library's fixed buffer holds";
        default: return "unknown status";
    }
}

extern "C" int grass_version(void) { return 200; }
