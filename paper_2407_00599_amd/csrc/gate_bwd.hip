// Backward of the gating function of Section II-A (linear layer + softmax + top-k), with the
// top-k selection held fixed.
//
//   gate_dlogits : one thread per token.  norm_topk: dl[e_j] = w_j (dw_j - sum_j' w_j' dw_j');
//                  otherwise dl[e] = sum_j dw_j p[e_j] (delta(e,e_j) - p[e]) with p = softmax(l).
//   gate_dx      : dx[t,m] (+)= sum_e dl[t,e] Wg[m,e].  A thread owns 8 consecutive m and keeps
//                  16 experts of Wg in registers while it walks over its tokens; dl rows are
//                  uniform per token.  Bound by the dx read/write.
//   gate_dwg_partial / gate_dwg_reduce : dWg[m,e] = sum_t x[t,m] dl[t,e] as per-token-chunk
//                  fp32 partial sums followed by a fixed-order fp64 reduction (no atomics, so
//                  the result is the same on every run).  dbias[e] = sum_t dl[t,e] rides along
//                  as an extra row m = M of the partials.
#include "common.h"

namespace {

using namespace moe;

constexpr int DX_TOK = 8;        // tokens per thread step in gate_dx
constexpr int DX_TOK_BLK = 8;    // tokens per block in gate_dx
// tokens per partial sum in gate_dwg_partial: at least 32, and at most 256 partial sums
inline int dwg_chunk(int64_t S) { const int64_t c = (S + 255) / 256; return (int)(c < 32 ? 32 : c); }

__global__ __launch_bounds__(256) void gate_dlogits(const float* __restrict__ dw, const float* __restrict__ w,
                                                    const int32_t* __restrict__ idx, const float* __restrict__ logits,
                                                    int64_t S, int E, int k, int norm_topk, float* __restrict__ dl) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= S) return;
  float wj[MOE_MAX_K], gj[MOE_MAX_K];
  int ej[MOE_MAX_K];
  float inner = 0.f;
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    wj[j] = 0.f; gj[j] = 0.f; ej[j] = -1;
    if (j < k) {
      wj[j] = w[t * k + j]; gj[j] = dw[t * k + j]; ej[j] = idx[t * k + j];
      inner = fmaf(wj[j], gj[j], inner);
    }
  }
  float mx = 0.f, den = 1.f;
  if (!norm_topk) {
    mx = logits[t * E];
    for (int e = 1; e < E; ++e) mx = fmaxf(mx, logits[t * E + e]);
    den = 0.f;
    for (int e = 0; e < E; ++e) den += expf(logits[t * E + e] - mx);
  }
  for (int e = 0; e < E; ++e) {
    float v = norm_topk ? 0.f : -(expf(logits[t * E + e] - mx) / den) * inner;
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (ej[j] == e) v += norm_topk ? wj[j] * (gj[j] - inner) : wj[j] * gj[j];
    dl[t * E + e] = v;
  }
}

template <bool BF16>
__device__ __forceinline__ void ld8g(const void* base, int64_t off, float* f) {
  if (BF16) {
    unpack_bf16x8(*reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(base) + off), f);
  } else {
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + off);
    const float4 a = p[0], b = p[1];
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
}
template <bool BF16>
__device__ __forceinline__ void st8g(void* base, int64_t off, const float* f) {
  if (BF16) {
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(base) + off) = pack_bf16x8(f);
  } else {
    float4* p = reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + off);
    p[0] = make_float4(f[0], f[1], f[2], f[3]);
    p[1] = make_float4(f[4], f[5], f[6], f[7]);
  }
}

// grid: (ceil(M/8/128), ceil(S/DX_TOK_BLK)); block 128 threads, thread -> 8 consecutive m.
template <bool BF16>
__global__ __launch_bounds__(128) void gate_dx(const float* __restrict__ dl, const float* __restrict__ Wg,
                                               void* __restrict__ dx, int64_t S, int M, int E, int accumulate) {
  const int m0 = (blockIdx.x * 128 + threadIdx.x) * 8;
  if (m0 >= M) return;
  const int64_t tb = (int64_t)blockIdx.y * DX_TOK_BLK;
  for (int64_t t0 = tb; t0 < tb + DX_TOK_BLK && t0 < S; t0 += DX_TOK) {
    float acc[DX_TOK][8];
#pragma unroll
    for (int i = 0; i < DX_TOK; ++i)
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[i][q] = 0.f;
    for (int e0 = 0; e0 < E; e0 += 16) {
      float wr[8][16];
#pragma unroll
      for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) wr[q][e] = (e0 + e < E) ? Wg[(int64_t)(m0 + q) * E + e0 + e] : 0.f;
#pragma unroll
      for (int i = 0; i < DX_TOK; ++i) {
        const int64_t t = t0 + i;
        if (t < S) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const float d = (e0 + e < E) ? dl[t * E + e0 + e] : 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[i][q] = fmaf(d, wr[q][e], acc[i][q]);
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < DX_TOK; ++i) {
      const int64_t t = t0 + i;
      if (t < S) {
        if (accumulate) {
          float old[8];
          ld8g<BF16>(dx, t * (int64_t)M + m0, old);
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[i][q] += old[q];
        }
        st8g<BF16>(dx, t * (int64_t)M + m0, acc[i]);
      }
    }
  }
}

// grid: (ceil(M/8/128), nchunk); partial[chunk][m][e] for m < M, plus row m = M for dbias.
template <bool BF16>
__global__ __launch_bounds__(128) void gate_dwg_partial(const void* __restrict__ x, const float* __restrict__ dl,
                                                        float* __restrict__ partial, int64_t S, int M, int E,
                                                        int chunk) {
  const int m0 = (blockIdx.x * 128 + threadIdx.x) * 8;
  const int64_t tb = (int64_t)blockIdx.y * chunk;
  const int64_t te = (tb + chunk < S) ? tb + chunk : S;
  float* out = partial + (int64_t)blockIdx.y * (M + 1) * E;
  if (m0 < M) {
    for (int e0 = 0; e0 < E; e0 += 16) {
      float acc[8][16];
#pragma unroll
      for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
#pragma unroll 4
      for (int64_t t = tb; t < te; ++t) {
        float xf[8];
        ld8g<BF16>(x, t * (int64_t)M + m0, xf);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float d = (e0 + e < E) ? dl[t * E + e0 + e] : 0.f;
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[q][e] = fmaf(xf[q], d, acc[q][e]);
        }
      }
#pragma unroll
      for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (e0 + e < E) out[(int64_t)(m0 + q) * E + e0 + e] = acc[q][e];
    }
  }
  if (blockIdx.x == 0) {  // bias row: column sums of dl over this chunk
    for (int e = threadIdx.x; e < E; e += 128) {
      float s = 0.f;
      for (int64_t t = tb; t < te; ++t) s += dl[t * E + e];
      out[(int64_t)M * E + e] = s;
    }
  }
}

__global__ __launch_bounds__(64) void gate_dwg_reduce(const float* __restrict__ partial, int nchunk, int M, int E,
                                                      float* __restrict__ dWg, float* __restrict__ dbias) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = (int64_t)(M + 1) * E;
  if (i >= n) return;
  // eight independent running sums keep eight loads in flight; the order of additions is fixed
  double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int c = 0;
  for (; c + 8 <= nchunk; c += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u) s[u] += (double)partial[(int64_t)(c + u) * n + i];
  }
  for (; c < nchunk; ++c) s[0] += (double)partial[(int64_t)c * n + i];
  const double t = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
  if (i < (int64_t)M * E) dWg[i] = (float)t;
  else if (dbias) dbias[i - (int64_t)M * E] = (float)t;
}

}  // namespace

extern "C" size_t moe_gate_bwd_workspace_bytes(int64_t S, int M, int E) {
  if (S < 1 || M < 1 || E < 1) return 0;
  const int chunk = dwg_chunk(S);
  const int64_t nchunk = (S + chunk - 1) / chunk;
  return moe::align_up((size_t)nchunk * (size_t)(M + 1) * E * sizeof(float), 256);
}

extern "C" int moe_gate_bwd(const float* dw, const float* w, const int32_t* idx, const float* logits, const void* x,
                            int x_dtype, const float* Wg, int64_t S, int M, int E, int k, int norm_topk,
                            float* dlogits, float* dWg, float* dgate_bias, void* dx, int dx_accumulate, void* ws,
                            size_t ws_bytes, void* stream) {
  if (int rc = moe::common_shape_check(S, M, E, k, 1)) return rc;
  MOE_REQUIRE(x_dtype == MOE_F32 || x_dtype == MOE_BF16, MOE_EINVAL);
  MOE_REQUIRE(norm_topk >= -1 && norm_topk <= 1, MOE_EINVAL);
  MOE_REQUIRE(dx_accumulate == 0 || dx_accumulate == 1, MOE_EINVAL);
  MOE_REQUIRE_PTR(dw); MOE_REQUIRE_PTR(w); MOE_REQUIRE_PTR(idx); MOE_REQUIRE_PTR(logits); MOE_REQUIRE_PTR(x);
  MOE_REQUIRE_PTR(Wg); MOE_REQUIRE_PTR(dlogits); MOE_REQUIRE_PTR(dWg); MOE_REQUIRE_PTR(dx);
  MOE_OPTIONAL_PTR(dgate_bias);
  const size_t need = moe_gate_bwd_workspace_bytes(S, M, E);
  MOE_REQUIRE(ws != nullptr && ws_bytes >= need, MOE_EWORKSPACE);
  MOE_REQUIRE(moe::aligned16(ws), MOE_EALIGN);
  const int norm = norm_topk < 0 ? (k >= 2 ? 1 : 0) : norm_topk;
  hipStream_t st = (hipStream_t)stream;
  const bool bf = x_dtype == MOE_BF16;
  hipLaunchKernelGGL(gate_dlogits, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, st, dw, w, idx, logits, S, E, k,
                     norm, dlogits);
  const unsigned gm = (unsigned)((M / 8 + 127) / 128);
  const dim3 grid_dx(gm, (unsigned)((S + DX_TOK_BLK - 1) / DX_TOK_BLK));
  if (bf) hipLaunchKernelGGL(gate_dx<true>, grid_dx, dim3(128), 0, st, dlogits, Wg, dx, S, M, E, dx_accumulate);
  else hipLaunchKernelGGL(gate_dx<false>, grid_dx, dim3(128), 0, st, dlogits, Wg, dx, S, M, E, dx_accumulate);
  const int chunk = dwg_chunk(S);
  const int nchunk = (int)((S + chunk - 1) / chunk);
  const dim3 grid_p(gm, (unsigned)nchunk);
  float* partial = (float*)ws;
  if (bf) hipLaunchKernelGGL(gate_dwg_partial<true>, grid_p, dim3(128), 0, st, x, dlogits, partial, S, M, E, chunk);
  else hipLaunchKernelGGL(gate_dwg_partial<false>, grid_p, dim3(128), 0, st, x, dlogits, partial, S, M, E, chunk);
  const int64_t n = (int64_t)(M + 1) * E;
  hipLaunchKernelGGL(gate_dwg_reduce, dim3((unsigned)((n + 63) / 64)), dim3(64), 0, st, partial, nchunk, M, E, dWg,
                     dgate_bias);
  return moe::check_launch();
}
