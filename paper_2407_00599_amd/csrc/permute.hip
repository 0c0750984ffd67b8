// Dispatch and combine of the MoE layer (Section II-A: G[i,:,:] holds the tokens of expert i;
// the expert outputs are combined back to token order) and the local sum of the N_ESP
// partial results that return through the EP&ESP-AlltoAll (Section III-C).
//
// All three kernels are row movers bound by HBM bandwidth.  They run in gather form: every
// output row is produced by exactly one wave, reading its source rows through the slot
// maps, so there are no atomics and no prior memset; 16-byte accesses per lane.
#include "common.h"

namespace {

using namespace moe;

// 8 consecutive elements as fp32
template <bool BF16>
__device__ __forceinline__ void ld8(const void* base, int64_t off, float* f) {
  if (BF16) {
    unpack_bf16x8(*reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(base) + off), f);
  } else {
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + off);
    const float4 a = p[0], b = p[1];
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
}
template <bool BF16>
__device__ __forceinline__ void st8(void* base, int64_t off, const float* f) {
  if (BF16) {
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(base) + off) = pack_bf16x8(f);
  } else {
    float4* p = reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + off);
    p[0] = make_float4(f[0], f[1], f[2], f[3]);
    p[1] = make_float4(f[4], f[5], f[6], f[7]);
  }
}

// buf[e, c, :] = (w?) * x[inv[e, c0 + c]/k, :]  or zeros, for the slots c0 <= c0 + c < c0 + Cr of every expert
// (buf is [E, Cr, M]; the whole buffer when c0 = 0 and Cr = C).  One wave per output row.
template <bool BF16>
__device__ __forceinline__ void dispatch_rows_body(int64_t blk, const void* __restrict__ x,
                                                   const int32_t* __restrict__ inv, const float* __restrict__ w,
                                                   void* __restrict__ buf, int64_t rows, int M, int k, int64_t C,
                                                   int64_t c0, int64_t Cr) {
  const int lane = threadIdx.x & 63;
  const int64_t row = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int64_t e = row / Cr;
  const int a = inv[e * C + c0 + (row - e * Cr)];
  const int64_t dst = row * (int64_t)M;
  if (a < 0) {
    const float z[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int m = lane * 8; m < M; m += 512) st8<BF16>(buf, dst + m, z);
    return;
  }
  const int64_t src = (int64_t)(a / k) * M;
  if (w == nullptr) {
    if (BF16) {
      for (int m = lane * 8; m < M; m += 512)
        *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(buf) + dst + m) =
            *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(x) + src + m);
    } else {
      for (int m = lane * 4; m < M; m += 256)
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(buf) + dst + m) =
            *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(x) + src + m);
    }
  } else {
    const float s = w[a];
    for (int m = lane * 8; m < M; m += 512) {
      float f[8];
      ld8<BF16>(x, src + m, f);
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] *= s;
      st8<BF16>(buf, dst + m, f);
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void dispatch_rows(const void* __restrict__ x, const int32_t* __restrict__ inv,
                                                     const float* __restrict__ w, void* __restrict__ buf,
                                                     int64_t rows, int M, int k, int64_t C, int64_t c0, int64_t Cr) {
  dispatch_rows_body<BF16>((int64_t)blockIdx.x, x, inv, w, buf, rows, M, k, C, c0, Cr);
}

// y[t,:] = sum_j w[t,j] * sum_p Yret[p, idx[t,j], slot[t,j], :].  One wave per token.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_rows(const void* __restrict__ Yret, const int32_t* __restrict__ idx,
                                                    const int32_t* __restrict__ slot, const float* __restrict__ w,
                                                    void* __restrict__ y, int64_t S, int M, int k, int64_t C,
                                                    int n_part, int64_t part_stride) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= S) return;
  int64_t src[MOE_MAX_K];
  float wt[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    src[j] = -1; wt[j] = 0.f;
    if (j < k) {
      const int c = slot[t * k + j];
      if (c >= 0) {
        src[j] = ((int64_t)idx[t * k + j] * C + c) * M;
        wt[j] = w ? w[t * k + j] : 1.f;
      }
    }
  }
  // two 512-element chunks per step: twice as many independent loads in flight per lane
  for (int m = lane * 8; m < M; m += 1024) {
    const bool two = m + 512 < M;
    float acc0[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float acc1[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
      if (j < k && src[j] >= 0) {
        float r0[8], r1[8];
        ld8<BF16>(Yret, src[j] + m, r0);
        if (two) ld8<BF16>(Yret, src[j] + m + 512, r1);
        for (int p = 1; p < n_part; ++p) {
          float q0[8], q1[8];
          ld8<BF16>(Yret, src[j] + m + p * part_stride, q0);
          if (two) ld8<BF16>(Yret, src[j] + m + 512 + p * part_stride, q1);
#pragma unroll
          for (int i = 0; i < 8; ++i) r0[i] += q0[i];
          if (two) {
#pragma unroll
            for (int i = 0; i < 8; ++i) r1[i] += q1[i];
          }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc0[i] = fmaf(wt[j], r0[i], acc0[i]);
        if (two) {
#pragma unroll
          for (int i = 0; i < 8; ++i) acc1[i] = fmaf(wt[j], r1[i], acc1[i]);
        }
      }
    }
    st8<BF16>(y, t * (int64_t)M + m, acc0);
    if (two) st8<BF16>(y, t * (int64_t)M + m + 512, acc1);
  }
}

// The common case (k <= 2 choices per token, 1, 2 or 4 partial sums per slot) with K and P fixed at
// compile time: all K * P * NCH row pieces of a step are requested before the first is used, NCH
// 512-element chunks per step so that about eight 16-byte loads per lane are in flight.
template <bool BF16>
struct Piece {   // 8 consecutive elements as loaded
  uint4 a, b;    // bf16: a only
};
// loaded with the non-temporal hint: each returned row is read exactly once (measured: 266 -> 234 us for
// 1.3 GB at S = 32768, M = 4096; the same hint on the store of y costs 4 %)
template <bool BF16>
__device__ __forceinline__ void ld_piece(Piece<BF16>& r, const void* base, int64_t off) {
  typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
  if (BF16) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(reinterpret_cast<const bf16_t*>(base) + off));
    r.a = make_uint4(v.x, v.y, v.z, v.w);
  } else {
    const u32x4_t* p = reinterpret_cast<const u32x4_t*>(reinterpret_cast<const float*>(base) + off);
    const u32x4_t v0 = __builtin_nontemporal_load(p), v1 = __builtin_nontemporal_load(p + 1);
    r.a = make_uint4(v0.x, v0.y, v0.z, v0.w); r.b = make_uint4(v1.x, v1.y, v1.z, v1.w);
  }
}
template <bool BF16>
__device__ __forceinline__ void piece_to_f32(const Piece<BF16>& r, float* f) {
  if (BF16) unpack_bf16x8(r.a, f);
  else {
    f[0] = __uint_as_float(r.a.x); f[1] = __uint_as_float(r.a.y); f[2] = __uint_as_float(r.a.z); f[3] = __uint_as_float(r.a.w);
    f[4] = __uint_as_float(r.b.x); f[5] = __uint_as_float(r.b.y); f[6] = __uint_as_float(r.b.z); f[7] = __uint_as_float(r.b.w);
  }
}
template <bool BF16, int K, int P>
__global__ __launch_bounds__(256) void combine_rows_kp(const void* __restrict__ Yret, const int32_t* __restrict__ idx,
                                                       const int32_t* __restrict__ slot, const float* __restrict__ w,
                                                       void* __restrict__ y, int64_t S, int M, int64_t C,
                                                       int64_t part_stride) {
  constexpr int NCH = (K * P >= 8) ? 1 : (K * P >= 4) ? 2 : 4;
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= S) return;
  int64_t src[K];
  float wt[K];
#pragma unroll
  for (int j = 0; j < K; ++j) {
    const int c = slot[t * K + j];
    src[j] = c >= 0 ? ((int64_t)idx[t * K + j] * C + c) * M : -1;
    wt[j] = (c >= 0) ? (w ? w[t * K + j] : 1.f) : 0.f;
  }
  for (int m0 = lane * 8; m0 < M; m0 += 512 * NCH) {
    Piece<BF16> raw[NCH][K][P];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
      for (int j = 0; j < K; ++j)
        if (src[j] >= 0 && m0 + 512 * c < M) {
#pragma unroll
          for (int p = 0; p < P; ++p) ld_piece<BF16>(raw[c][j][p], Yret, src[j] + p * part_stride + m0 + 512 * c);
        }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      if (m0 + 512 * c >= M) break;
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < K; ++j)
        if (src[j] >= 0) {
          float r[8];
          piece_to_f32<BF16>(raw[c][j][0], r);
#pragma unroll
          for (int p = 1; p < P; ++p) {
            float q[8];
            piece_to_f32<BF16>(raw[c][j][p], q);
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] += q[i];
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[i] = fmaf(wt[j], r[i], acc[i]);
        }
      st8<BF16>(y, t * (int64_t)M + m0 + 512 * c, acc);
    }
  }
}

// dw[t,j] = <dy[t,:], sum_p Yret[p, idx, slot, :]>, 0 for dropped choices.  One wave per token.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_dw(const void* __restrict__ dy, const void* __restrict__ Yret,
                                                  const int32_t* __restrict__ idx, const int32_t* __restrict__ slot,
                                                  float* __restrict__ dw, int64_t S, int M, int k, int64_t C,
                                                  int n_part, int64_t part_stride) {
  const int lane = threadIdx.x & 63;
  const int64_t t = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= S) return;
  int64_t src[MOE_MAX_K];
  float dot[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    src[j] = -1; dot[j] = 0.f;
    if (j < k) {
      const int c = slot[t * k + j];
      if (c >= 0) src[j] = ((int64_t)idx[t * k + j] * C + c) * M;
    }
  }
  // dy is read once per chunk and dotted with the rows of all surviving choices
  for (int m = lane * 8; m < M; m += 512) {
    float g[8];
    ld8<BF16>(dy, t * (int64_t)M + m, g);
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
      if (j < k && src[j] >= 0) {
        float r[8];
        ld8<BF16>(Yret, src[j] + m, r);
        for (int p = 1; p < n_part; ++p) {
          float q[8];
          ld8<BF16>(Yret, src[j] + m + p * part_stride, q);
#pragma unroll
          for (int i = 0; i < 8; ++i) r[i] += q[i];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) dot[j] = fmaf(g[i], r[i], dot[j]);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    if (j < k) {
      float d = dot[j];
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) d += __shfl_xor(d, o, 64);
      if (lane == 0) dw[t * k + j] = d;
    }
  }
}

template <bool BF16, int K, int P>
__device__ __forceinline__ void combine_dw_kp_body(int64_t blk, const void* __restrict__ dy, const void* __restrict__ Yret,
                                                   const int32_t* __restrict__ idx, const int32_t* __restrict__ slot,
                                                   float* __restrict__ dw, int64_t S, int M, int64_t C,
                                                   int64_t part_stride) {
  constexpr int NCH = (K * P >= 8) ? 1 : (K * P >= 4) ? 2 : 4;
  const int lane = threadIdx.x & 63;
  const int64_t t = blk * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= S) return;
  int64_t src[K];
  float dot[K];
#pragma unroll
  for (int j = 0; j < K; ++j) {
    const int c = slot[t * K + j];
    src[j] = c >= 0 ? ((int64_t)idx[t * K + j] * C + c) * M : -1;
    dot[j] = 0.f;
  }
  for (int m0 = lane * 8; m0 < M; m0 += 512 * NCH) {
    Piece<BF16> raw[NCH][K][P], gr[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
      if (m0 + 512 * c < M) {
        ld_piece<BF16>(gr[c], dy, t * (int64_t)M + m0 + 512 * c);
#pragma unroll
        for (int j = 0; j < K; ++j)
          if (src[j] >= 0) {
#pragma unroll
            for (int p = 0; p < P; ++p) ld_piece<BF16>(raw[c][j][p], Yret, src[j] + p * part_stride + m0 + 512 * c);
          }
      }
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      if (m0 + 512 * c >= M) break;
      float g[8];
      piece_to_f32<BF16>(gr[c], g);
#pragma unroll
      for (int j = 0; j < K; ++j)
        if (src[j] >= 0) {
          float r[8];
          piece_to_f32<BF16>(raw[c][j][0], r);
#pragma unroll
          for (int p = 1; p < P; ++p) {
            float q[8];
            piece_to_f32<BF16>(raw[c][j][p], q);
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] += q[i];
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) dot[j] = fmaf(g[i], r[i], dot[j]);
        }
    }
  }
#pragma unroll
  for (int j = 0; j < K; ++j) {
    float d = dot[j];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) d += __shfl_xor(d, o, 64);
    if (lane == 0) dw[t * K + j] = d;
  }
}

// The whole combine backward in one launch: the first nb_rows workgroups write dYret (the weighted
// dispatch of dy), the others the weight gradients.
template <bool BF16, int K, int P>
__global__ __launch_bounds__(256) void combine_bwd_kp(const void* __restrict__ dy, const void* __restrict__ Yret,
                                                      const int32_t* __restrict__ idx, const int32_t* __restrict__ slot,
                                                      const int32_t* __restrict__ inv, const float* __restrict__ w,
                                                      void* __restrict__ dYret, float* __restrict__ dw, int64_t S, int M,
                                                      int64_t C, int64_t part_stride, int64_t rows, int64_t nb_rows) {
  const int64_t b = (int64_t)blockIdx.x;
  if (b < nb_rows) dispatch_rows_body<BF16>(b, dy, inv, w, dYret, rows, M, K, C, (int64_t)0, C);
  else combine_dw_kp_body<BF16, K, P>(b - nb_rows, dy, Yret, idx, slot, dw, S, M, C, part_stride);
}

}  // namespace

extern "C" int moe_dispatch_slots(const void* x, int dtype, int64_t S, int M, int E, int k, int64_t C, int64_t c0,
                                  int64_t c1, const int32_t* inv, const float* w, void* buf, void* stream) {
  if (int rc = moe::common_shape_check(S, M, E, k, C)) return rc;
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_EINVAL);
  MOE_REQUIRE(c0 >= 0 && c0 < c1 && c1 <= C, MOE_EINVAL);
  MOE_REQUIRE_PTR(x); MOE_REQUIRE_PTR(inv); MOE_REQUIRE_PTR(buf);
  MOE_OPTIONAL_PTR(w);
  const int64_t Cr = c1 - c0;
  const int64_t rows = (int64_t)E * Cr;
  const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MOE_BF16) hipLaunchKernelGGL(dispatch_rows<true>, grid, block, 0, st, x, inv, w, buf, rows, M, k, C, c0, Cr);
  else hipLaunchKernelGGL(dispatch_rows<false>, grid, block, 0, st, x, inv, w, buf, rows, M, k, C, c0, Cr);
  return moe::check_launch();
}

extern "C" int moe_dispatch(const void* x, int dtype, int64_t S, int M, int E, int k, int64_t C,
                            const int32_t* inv, const float* w, void* buf, void* stream) {
  if (int rc = moe::common_shape_check(S, M, E, k, C)) return rc;
  return moe_dispatch_slots(x, dtype, S, M, E, k, C, 0, C, inv, w, buf, stream);
}

extern "C" int moe_combine_fwd(const void* Yret, int dtype, int n_part, int64_t S, int M, int E, int k, int64_t C,
                               const int32_t* idx, const int32_t* slot, const float* w, void* y, void* stream) {
  if (int rc = moe::common_shape_check(S, M, E, k, C)) return rc;
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_EINVAL);
  MOE_REQUIRE(n_part >= 1 && n_part <= 64, MOE_EINVAL);
  MOE_REQUIRE_PTR(Yret); MOE_REQUIRE_PTR(idx); MOE_REQUIRE_PTR(slot); MOE_REQUIRE_PTR(y);
  MOE_OPTIONAL_PTR(w);
  const dim3 grid((unsigned)((S + 3) / 4)), block(256);
  const int64_t ps = (int64_t)E * C * M;
  hipStream_t st = (hipStream_t)stream;
  const bool bf = dtype == MOE_BF16;
#define COMBINE_KP(K_, P_)                                                                                          \
  if (k == K_ && n_part == P_) {                                                                                    \
    if (bf) hipLaunchKernelGGL((combine_rows_kp<true, K_, P_>), grid, block, 0, st, Yret, idx, slot, w, y, S, M, C, ps); \
    else hipLaunchKernelGGL((combine_rows_kp<false, K_, P_>), grid, block, 0, st, Yret, idx, slot, w, y, S, M, C, ps);   \
    return moe::check_launch();                                                                                     \
  }
  COMBINE_KP(1, 1) COMBINE_KP(1, 2) COMBINE_KP(1, 4) COMBINE_KP(2, 1) COMBINE_KP(2, 2) COMBINE_KP(2, 4)
#undef COMBINE_KP
  if (bf) hipLaunchKernelGGL(combine_rows<true>, grid, block, 0, st, Yret, idx, slot, w, y, S, M, k, C, n_part, ps);
  else hipLaunchKernelGGL(combine_rows<false>, grid, block, 0, st, Yret, idx, slot, w, y, S, M, k, C, n_part, ps);
  return moe::check_launch();
}

extern "C" int moe_combine_bwd(const void* dy, const void* Yret, int dtype, int n_part, int64_t S, int M, int E,
                               int k, int64_t C, const int32_t* idx, const int32_t* slot, const int32_t* inv,
                               const float* w, void* dYret, float* dw, void* stream) {
  if (int rc = moe::common_shape_check(S, M, E, k, C)) return rc;
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_EINVAL);
  MOE_REQUIRE(n_part >= 1 && n_part <= 64, MOE_EINVAL);
  MOE_REQUIRE_PTR(dy); MOE_REQUIRE_PTR(Yret); MOE_REQUIRE_PTR(idx); MOE_REQUIRE_PTR(slot); MOE_REQUIRE_PTR(inv);
  MOE_REQUIRE_PTR(w); MOE_OPTIONAL_PTR(dYret); MOE_REQUIRE_PTR(dw);
  hipStream_t st = (hipStream_t)stream;
  const int64_t rows = (int64_t)E * C;
  const int64_t ps = rows * M;
  const dim3 block(256), grid_r((unsigned)((rows + 3) / 4)), grid_t((unsigned)((S + 3) / 4));
  const bool bf = dtype == MOE_BF16;
  const int64_t nb_rows = dYret ? (int64_t)grid_r.x : 0;
  const dim3 grid_b((unsigned)(nb_rows + grid_t.x));
#define COMBINE_DW_KP(K_, P_)                                                                                          \
  if (k == K_ && n_part == P_) {                                                                                       \
    if (bf) hipLaunchKernelGGL((combine_bwd_kp<true, K_, P_>), grid_b, block, 0, st, dy, Yret, idx, slot, inv, w, dYret, dw, \
                               S, M, C, ps, rows, nb_rows);                                                            \
    else hipLaunchKernelGGL((combine_bwd_kp<false, K_, P_>), grid_b, block, 0, st, dy, Yret, idx, slot, inv, w, dYret, dw,   \
                            S, M, C, ps, rows, nb_rows);                                                               \
    return moe::check_launch();                                                                                        \
  }
  COMBINE_DW_KP(1, 1) COMBINE_DW_KP(1, 2) COMBINE_DW_KP(1, 4) COMBINE_DW_KP(2, 1) COMBINE_DW_KP(2, 2) COMBINE_DW_KP(2, 4)
#undef COMBINE_DW_KP
  if (dYret) {
    if (bf) hipLaunchKernelGGL(dispatch_rows<true>, grid_r, block, 0, st, dy, inv, w, dYret, rows, M, k, C, (int64_t)0, C);
    else hipLaunchKernelGGL(dispatch_rows<false>, grid_r, block, 0, st, dy, inv, w, dYret, rows, M, k, C, (int64_t)0, C);
  }
  if (bf) hipLaunchKernelGGL(combine_dw<true>, grid_t, block, 0, st, dy, Yret, idx, slot, dw, S, M, k, C, n_part, ps);
  else hipLaunchKernelGGL(combine_dw<false>, grid_t, block, 0, st, dy, Yret, idx, slot, dw, S, M, k, C, n_part, ps);
  return moe::check_launch();
}
