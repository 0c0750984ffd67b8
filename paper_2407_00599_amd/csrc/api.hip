// Host-only entry points of libparm_moe: error strings, ABI version, expert capacity.
#include <cmath>

#include "common.h"

extern "C" const char* moe_strerror(int err) {
  switch (err) {
    case MOE_OK: return "ok";
    case MOE_EINVAL: return "invalid argument (shape or index out of range)";
    case MOE_EUNSUPPORTED: return "shape or type outside the limits of this build";
    case MOE_EALIGN: return "pointer is not 16-byte aligned";
    case MOE_ELAUNCH: return "HIP reported an error while enqueuing";
    case MOE_EWORKSPACE: return "workspace missing or too small";
    case MOE_ENULL: return "required pointer is NULL";
    case MOE_ESCRATCH: return "problem exceeds the library's static scratch array";
    default: return "unknown error code";
  }
}

extern "C" int moe_abi_version(void) { return 6; }

// Section II-A: T := k * f * B * L / E, here for the S tokens this rank gates; rounded up.
extern "C" int64_t moe_capacity(int64_t S, int E, int k, double f) {
  if (S < 1 || E < 1 || k < 1 || k > E || !(f > 0.0) || !std::isfinite(f)) return -1;
  const double t = ((double)(k * S) * f) / (double)E;
  const double c = std::ceil(t);
  if (c >= 2147483647.0) return -1;
  return c < 1.0 ? 1 : (int64_t)c;
}
