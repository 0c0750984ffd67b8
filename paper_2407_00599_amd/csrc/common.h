// Internal helpers shared by the HIP sources of libparm_moe (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "parm_moe.h"

#define MOE_MAX_K 8
#define MOE_MAX_E 256

typedef uint16_t bf16_t;  // raw bfloat16 bits as stored in memory

namespace moe {

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; inputs on this path are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two floats -> packed bf16 pair with the hardware converter (v_cvt_pk_bf16_f32, round-to-nearest-even)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ void unpack_bf16x8(const uint4& v, float* f) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

__device__ __forceinline__ uint4 pack_bf16x8(const float* f) {
  uint4 v;
  v.x = pack_bf16x2(f[0], f[1]); v.y = pack_bf16x2(f[2], f[3]);
  v.z = pack_bf16x2(f[4], f[5]); v.w = pack_bf16x2(f[6], f[7]);
  return v;
}

// exact (erf) GeLU and its derivative, fp32
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }
__device__ __forceinline__ void gelu_and_grad(float z, float& g, float& dg) {
  const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
  g = z * cdf;
  dg = cdf + z * 0.39894228040143267794f * __expf(-0.5f * z * z);
}

// ---- host-side argument checks ----
inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

#define MOE_REQUIRE(cond, err) do { if (!(cond)) return (err); } while (0)
#define MOE_REQUIRE_PTR(p) do { if ((p) == nullptr) return MOE_ENULL; if (!moe::aligned16(p)) return MOE_EALIGN; } while (0)
#define MOE_OPTIONAL_PTR(p) do { if ((p) != nullptr && !moe::aligned16(p)) return MOE_EALIGN; } while (0)

inline int check_launch() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ELAUNCH; }

inline int common_shape_check(int64_t S, int M, int E, int k, int64_t C) {
  if (S < 1 || M < 1 || E < 1 || k < 1 || C < 1) return MOE_EINVAL;
  if (k > E) return MOE_EINVAL;
  if (k > MOE_MAX_K || E > MOE_MAX_E) return MOE_EUNSUPPORTED;
  if (M % 8 != 0) return MOE_EUNSUPPORTED;
  if (S * (int64_t)k >= (int64_t)1 << 31 || (int64_t)E * C >= (int64_t)1 << 31) return MOE_EUNSUPPORTED;
  return MOE_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace moe
