// Error reporting of the C ABI.
#include "common.h"

namespace imu {
thread_local int g_last_hip_error = 0;
}

extern "C" const char *imunpack_strerror(int code) {
    switch (code) {
        case IMUNPACK_OK: return "ok";
        case IMUNPACK_EINVAL: return "invalid argument";
        case IMUNPACK_ERANGE: return "value or accumulator bound out of range";
        case IMUNPACK_ENOMEM: return "out of memory";
        case IMUNPACK_EHIP: return "HIP runtime error";
        case IMUNPACK_ESMALL: return "buffer too small";
        default: return "unknown error";
    }
}

extern "C" int imunpack_last_hip_error(void) { return imu::g_last_hip_error; }
