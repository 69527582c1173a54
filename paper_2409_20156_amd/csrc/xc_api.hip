// Status strings and per-thread HIP error of the C ABI.
#include "xc_common.h"

namespace xc {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = static_cast<int>(e); }
}  // namespace xc

extern "C" const char* xc_strerror(int status) {
    switch (status) {
        case XC_OK: return "ok";
        case XC_EINVAL: return "invalid argument (null or misaligned pointer, bad enum)";
        case XC_ESHAPE: return "unsupported or inconsistent sizes";
        case XC_EWORKSPACE: return "workspace too small";
        case XC_EHIP: return "HIP runtime error (see xc_last_hip_error)";
        default: return "unknown status";
    }
}

extern "C" int xc_last_hip_error(void) { return xc::g_last_hip_error; }

extern "C" int xc_version(void) { return 1; }
