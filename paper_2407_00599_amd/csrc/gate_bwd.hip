// Backward of the gating function of Section II-A (linear layer + softmax + top-k), with the
// top-k selection held fixed.
//
//   E <= 16 : gate_bwd_fused (dlogits, dx and the dWg partial sums in one kernel) + gate_dwg_reduce.
//   E  > 16 : gate_dlogits (one thread per token; norm_topk: dl[e_j] = w_j (dw_j - sum_j' w_j' dw_j'),
//             otherwise dl[e] = sum_j dw_j p[e_j] (delta(e,e_j) - p[e]) with p = softmax(l)),
//             gate_dx_wide (dx[t,m] (+)= sum_e dl[t,e] Wg[m,e]), gate_dwg_wide + gate_dwg_reduce.
//   dWg[m,e] = sum_t x[t,m] dl[t,e] is formed as per-token-chunk fp32 partial sums followed by a
//   fixed-order fp64 reduction (no atomics, so the result is the same on every run); dbias[e] =
//   sum_t dl[t,e] rides along as an extra row m = M of the partials.
#include "common.h"

namespace {

using namespace moe;

// tokens per dWg partial sum: a multiple of 8, at least 8, and at most 256 partial sums
// (more than 16 experts: at most 64 partial sums of at least 64 tokens, the partials being E/8 times larger)
inline int dwg_chunk(int64_t S, int E) {
  const int64_t parts = E <= 16 ? 256 : 64, least = E <= 16 ? 8 : 64;
  const int64_t c = (S + parts - 1) / parts;
  return (int)(c < least ? least : (c + 7) / 8 * 8);
}

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

// dWg[i] = sum over the chunks of partial[chunk][i], in a fixed order: the four waves of a block take
// every fourth group of four chunks each (four running fp64 sums apiece, so sixteen loads are in flight
// per output), and wave 0 adds the four results.
__global__ __launch_bounds__(256) void gate_dwg_reduce(const float* __restrict__ partial, int nchunk, int M, int E,
                                                       float* __restrict__ dWg, float* __restrict__ dbias) {
  __shared__ double red[4][64];
  const int o = threadIdx.x & 63, gq = threadIdx.x >> 6;
  const int64_t i = (int64_t)blockIdx.x * 64 + o;
  const int64_t n = (int64_t)(M + 1) * E;
  double s[4] = {0, 0, 0, 0};
  if (i < n) {
    int c = gq * 4;
    for (; c + 20 <= nchunk; c += 32) {   // two of this wave's groups at a time: eight loads in flight
      float v[8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        v[u] = partial[(int64_t)(c + u) * n + i];
        v[4 + u] = partial[(int64_t)(c + 16 + u) * n + i];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) s[u] += (double)v[u];
#pragma unroll
      for (int u = 0; u < 4; ++u) s[u] += (double)v[4 + u];
    }
    for (; c < nchunk; c += 16) {
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c + u < nchunk) s[u] += (double)partial[(int64_t)(c + u) * n + i];
    }
  }
  red[gq][o] = (s[0] + s[1]) + (s[2] + s[3]);
  __syncthreads();
  if (gq == 0 && i < n) {
    const double t = (red[0][o] + red[1][o]) + (red[2][o] + red[3][o]);
    if (i < (int64_t)M * E) dWg[i] = (float)t;
    else if (dbias) dbias[i - (int64_t)M * E] = (float)t;
  }
}

// ---------------------------------------------------------------------------------------------
// E <= 16: the whole gate backward except the final reduction in ONE kernel.  A block owns one
// chunk of tokens (the unit of a dWg partial sum) and NTHR * 4 columns of M (one wave, 256 columns,
// for up to 8 experts: many small blocks hide each other's phases; two waves for up to 16); a
// thread owns 4 consecutive columns, so that its slice of Wg and its dWg accumulators fit in registers.  Sixteen tokens at a time, sixteen threads compute the
// dlogits rows into LDS (column block 0 also stores them); then every thread reads its x and old
// dx pieces of those tokens once and uses them twice:
//     dWg partial[e][q] += x[t, q] dl[t, e]        dx[t, q] (+)= sum_e dl[t, e] Wg[q, e]
// The partial sums leave through LDS so that [m][e] rows are written contiguously.
// ---------------------------------------------------------------------------------------------
constexpr int FT = 16;   // tokens per dlogits stage
template <bool BF16, int N>
__device__ __forceinline__ void ldn(const void* base, int64_t off, float* f) {
  if (N == 8) { ld8g<BF16>(base, off, f); return; }
  if (BF16) {
    const uint2 v = *reinterpret_cast<const uint2*>(reinterpret_cast<const bf16_t*>(base) + off);
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  } else {
    const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + off);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
  }
}
template <bool BF16, int N>
__device__ __forceinline__ void stn(void* base, int64_t off, const float* f) {
  if (N == 8) { st8g<BF16>(base, off, f); return; }
  if (BF16) {
    *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(base) + off) = make_uint2(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]));
  } else {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + off) = make_float4(f[0], f[1], f[2], f[3]);
  }
}

// raw (unconverted) CPT elements of a row: requested for all tokens of a stage first, converted when used
template <bool BF16, int CPT>
struct RawRow {
  uint32_t r[BF16 ? CPT / 2 : CPT];
  __device__ __forceinline__ void load(const void* base, int64_t off) {
    constexpr int NB = (BF16 ? CPT / 2 : CPT) * 4;   // bytes: 8, 16 or 32
    const char* p = reinterpret_cast<const char*>(base) + off * (BF16 ? 2 : 4);
    if (NB == 8) { const uint2 v = *reinterpret_cast<const uint2*>(p); r[0] = v.x; r[1] = v.y; }
    else {
#pragma unroll
      for (int i = 0; i < NB / 16; ++i) {
        const uint4 v = reinterpret_cast<const uint4*>(p)[i];
        r[4 * i] = v.x; r[4 * i + 1] = v.y; r[4 * i + 2] = v.z; r[4 * i + 3] = v.w;
      }
    }
  }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int i = 0; i < (BF16 ? CPT / 2 : CPT); ++i) r[i] = 0u;
  }
  __device__ __forceinline__ float get(int q) const {
    if (BF16) return __uint_as_float((q & 1) ? (r[q >> 1] & 0xFFFF0000u) : (r[q >> 1] << 16));
    return __uint_as_float(r[q]);
  }
};

template <bool BF16, int EC, int CPT, int NTHR>
__global__ __launch_bounds__(NTHR) void gate_bwd_fused(const float* __restrict__ dw, const float* __restrict__ w,
                                                       const int32_t* __restrict__ idx, const float* __restrict__ logits,
                                                       const void* __restrict__ x, const float* __restrict__ Wg,
                                                       int64_t S, int M, int E, int k, int norm_topk, int chunk,
                                                       float* __restrict__ dl_out, void* __restrict__ dx, int accumulate,
                                                       float* __restrict__ partial) {
  constexpr int MT = NTHR * CPT, PITCH = MT + 8;
  __shared__ __attribute__((aligned(16))) float outs[EC * PITCH];
  __shared__ __attribute__((aligned(16))) float dls[FT * EC];
  const int tid = threadIdx.x;
  const int mb = blockIdx.x * MT, ml = tid * CPT, m0 = mb + ml;
  const bool mok = m0 < M;
  const int64_t tb = (int64_t)blockIdx.y * chunk;
  const int64_t te = (tb + chunk < S) ? tb + chunk : S;
  float* out = partial + (int64_t)blockIdx.y * (M + 1) * E;

  float wr[CPT][EC], acc[EC][CPT];
#pragma unroll
  for (int q = 0; q < CPT; ++q)
#pragma unroll
    for (int e = 0; e < EC; ++e) {
      wr[q][e] = (mok && e < E) ? Wg[(int64_t)(m0 + q) * E + e] : 0.f;
      acc[e][q] = 0.f;
    }
  float colsum = 0.f;   // thread e < E of column block 0 sums dl[:, e] for the bias row

  for (int64_t t0 = tb; t0 < te; t0 += FT) {
    const int nt = (int)((te - t0 < FT) ? te - t0 : FT);
    // the stage's x and old dx pieces are requested before the dlogits rows are worked out
    RawRow<BF16, CPT> xr[FT], dr[FT];
#pragma unroll
    for (int u = 0; u < FT; ++u) {
      if (mok && u < nt) xr[u].load(x, (t0 + u) * (int64_t)M + m0); else xr[u].zero();
      if (mok && u < nt && accumulate) dr[u].load(dx, (t0 + u) * (int64_t)M + m0); else dr[u].zero();
    }
    __syncthreads();   // the previous stage's dl rows are consumed
    if (tid < FT) {
      const int64_t t = t0 + tid;
      float row[EC];
#pragma unroll
      for (int e = 0; e < EC; ++e) row[e] = 0.f;
      if (t < te) {
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
#pragma unroll
        for (int e = 0; e < EC; ++e) {
          if (e < E) {
            float v = norm_topk ? 0.f : -(expf(logits[t * E + e] - mx) / den) * inner;
#pragma unroll
            for (int j = 0; j < MOE_MAX_K; ++j)
              if (ej[j] == e) v += norm_topk ? wj[j] * (gj[j] - inner) : wj[j] * gj[j];
            row[e] = v;
            if (blockIdx.x == 0) dl_out[t * E + e] = v;
          }
        }
      }
#pragma unroll
      for (int e = 0; e < EC; ++e) dls[tid * EC + e] = row[e];
    }
    __syncthreads();
    if (blockIdx.x == 0 && tid < EC)
      for (int t = 0; t < FT; ++t) colsum += dls[t * EC + tid];
    if (mok) {
#pragma unroll
      for (int u = 0; u < FT; ++u) {
        float xv[CPT], dv[CPT];
#pragma unroll
        for (int q = 0; q < CPT; ++q) { xv[q] = xr[u].get(q); dv[q] = dr[u].get(q); }
#pragma unroll
        for (int e4 = 0; e4 < EC; e4 += 4) {
          const float4 d4 = *reinterpret_cast<const float4*>(&dls[u * EC + e4]);
          const float d[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
              acc[e4 + v][q] = fmaf(xv[q], d[v], acc[e4 + v][q]);
              dv[q] = fmaf(d[v], wr[q][e4 + v], dv[q]);
            }
        }
        if (u < nt) stn<BF16, CPT>(dx, (t0 + u) * (int64_t)M + m0, dv);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < EC; ++e)
#pragma unroll
    for (int q = 0; q < CPT; q += 4)
      *reinterpret_cast<float4*>(&outs[e * PITCH + ml + q]) = make_float4(acc[e][q], acc[e][q + 1], acc[e][q + 2], acc[e][q + 3]);
  __syncthreads();
  for (int i = tid; i < MT * EC; i += NTHR) {
    const int m = i / EC, e = i - m * EC;
    if (mb + m < M && e < E) out[(int64_t)(mb + m) * E + e] = outs[e * PITCH + m];
  }
  if (blockIdx.x == 0 && tid < E && tid < EC) out[(int64_t)M * E + tid] = colsum;
}

// ---------------------------------------------------------------------------------------------
// E > 16.  The two products are small-K / small-N GEMMs on the vector ALUs with everything shared
// through LDS, experts taken 32 (dx) or 64 (dWg) at a time.
//
// gate_dx_wide: a block owns 64 tokens x 256 columns; thread = 4 columns x 16 tokens (64 fp32
// accumulators that stay in registers across the expert chunks).  Per chunk the Wg slab goes to LDS
// transposed, [e][column] with pitch 260, so a thread reads its 4 columns of an expert with one 16-byte
// access and consecutive lanes are contiguous; dl rows are read as wave-wide broadcasts.
// ---------------------------------------------------------------------------------------------
constexpr int WX_EB = 32, WX_TOK = 64, WX_COLS = 256, WX_PITCH = WX_COLS + 4;
template <bool BF16>
__global__ __launch_bounds__(256) void gate_dx_wide(const float* __restrict__ dl, const float* __restrict__ Wg,
                                                    void* __restrict__ dx, int64_t S, int M, int E, int accumulate) {
  __shared__ __attribute__((aligned(16))) float wgs[WX_EB * WX_PITCH];
  __shared__ __attribute__((aligned(16))) float dls[WX_TOK * WX_EB];
  const int tid = threadIdx.x, cg = tid & 63, tg = tid >> 6;
  const int cb = blockIdx.x * WX_COLS, c0 = cb + cg * 4;
  const int64_t tb = (int64_t)blockIdx.y * WX_TOK, t0 = tb + tg * 16;
  const bool cok = c0 < M;     // M is a multiple of 8, so 4 columns are in or out together
  float acc[16][4];
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    if (accumulate && cok && t0 + t < S) {
      ldn<BF16, 4>(dx, (t0 + t) * (int64_t)M + c0, acc[t]);
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[t][q] = 0.f;
    }
  }
  for (int ec = 0; ec < E; ec += WX_EB) {
    __syncthreads();
    for (int i = tid; i < WX_COLS * WX_EB; i += 256) {      // Wg[cb + c][ec + e], read along e
      const int c = i / WX_EB, e = i - c * WX_EB;
      wgs[e * WX_PITCH + c] = (cb + c < M && ec + e < E) ? Wg[(int64_t)(cb + c) * E + ec + e] : 0.f;
    }
    for (int i = tid; i < WX_TOK * WX_EB; i += 256) {
      const int t = i / WX_EB, e = i - t * WX_EB;
      dls[i] = (tb + t < S && ec + e < E) ? dl[(tb + t) * E + ec + e] : 0.f;
    }
    __syncthreads();
#pragma unroll 2
    for (int e4 = 0; e4 < WX_EB; e4 += 4) {
      float4 wv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) wv[j] = *reinterpret_cast<const float4*>(&wgs[(e4 + j) * WX_PITCH + cg * 4]);
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const float4 d = *reinterpret_cast<const float4*>(&dls[(tg * 16 + t) * WX_EB + e4]);
        const float dv[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[t][0] = fmaf(dv[j], wv[j].x, acc[t][0]);
          acc[t][1] = fmaf(dv[j], wv[j].y, acc[t][1]);
          acc[t][2] = fmaf(dv[j], wv[j].z, acc[t][2]);
          acc[t][3] = fmaf(dv[j], wv[j].w, acc[t][3]);
        }
      }
    }
  }
  if (cok) {
#pragma unroll
    for (int t = 0; t < 16; ++t)
      if (t0 + t < S) stn<BF16, 4>(dx, (t0 + t) * (int64_t)M + c0, acc[t]);
  }
}

// gate_dwg_wide: a block owns one token chunk x 256 columns x 64 experts (grid.z walks the expert
// blocks); thread = 4 columns x 16 experts (64 accumulators).  16 tokens at a time: their x pieces
// are requested first, the dl rows staged in LDS and read as broadcasts (a wave shares its 16 experts).
// partial[chunk][m][e] for m < M, plus row m = M (column sums of dl) for the bias gradient.
template <bool BF16>
__global__ __launch_bounds__(256) void gate_dwg_wide(const void* __restrict__ x, const float* __restrict__ dl,
                                                     float* __restrict__ partial, int64_t S, int M, int E, int chunk) {
  __shared__ __attribute__((aligned(16))) float dls[16 * 64];
  const int tid = threadIdx.x, cg = tid & 63, eg = tid >> 6;
  const int c0 = blockIdx.x * 256 + cg * 4;
  const int eb = blockIdx.z * 64;
  const bool cok = c0 < M;
  const int64_t tb = (int64_t)blockIdx.y * chunk;
  const int64_t te = (tb + chunk < S) ? tb + chunk : S;
  float* out = partial + (int64_t)blockIdx.y * (M + 1) * E;
  float acc[16][4];
#pragma unroll
  for (int j = 0; j < 16; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[j][q] = 0.f;
  float colsum = 0.f;
  for (int64_t t0 = tb; t0 < te; t0 += 16) {
    RawRow<BF16, 4> xr[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      if (cok && t0 + u < te) xr[u].load(x, (t0 + u) * (int64_t)M + c0); else xr[u].zero();
    }
    __syncthreads();
    for (int i = tid; i < 16 * 64; i += 256) {
      const int t = i >> 6, e = i & 63;
      dls[i] = (t0 + t < te && eb + e < E) ? dl[(t0 + t) * E + eb + e] : 0.f;
    }
    __syncthreads();
    if (blockIdx.x == 0 && tid < 64)
      for (int t = 0; t < 16; ++t) colsum += dls[t * 64 + tid];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const float xv[4] = {xr[u].get(0), xr[u].get(1), xr[u].get(2), xr[u].get(3)};
#pragma unroll
      for (int j4 = 0; j4 < 16; j4 += 4) {
        const float4 d = *reinterpret_cast<const float4*>(&dls[u * 64 + eg * 16 + j4]);
        const float dv[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[j4 + jj][q] = fmaf(xv[q], dv[jj], acc[j4 + jj][q]);
      }
    }
  }
  if (cok) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int e = eb + eg * 16 + j;
        if (e < E) out[(int64_t)(c0 + q) * E + e] = acc[j][q];
      }
  }
  if (blockIdx.x == 0 && tid < 64 && eb + tid < E) out[(int64_t)M * E + eb + tid] = colsum;
}

}  // namespace

extern "C" size_t moe_gate_bwd_workspace_bytes(int64_t S, int M, int E) {
  if (S < 1 || M < 1 || E < 1) return 0;
  const int chunk = dwg_chunk(S, E);
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
  const int64_t n = (int64_t)(M + 1) * E;
  if (E <= 16) {   // one fused kernel, then the reduction of the partial sums
    const int chunk = dwg_chunk(S, E);
    const int nchunk = (int)((S + chunk - 1) / chunk);
    float* partial = (float*)ws;
    const int cols = E <= 8 ? 64 * 4 : 128 * 4;   // columns per block
    const dim3 grid((unsigned)((M + cols - 1) / cols), (unsigned)nchunk);
#define MOE_FUSED(BF, EC, CPT, NT) hipLaunchKernelGGL((gate_bwd_fused<BF, EC, CPT, NT>), grid, dim3(NT), 0, st, dw, w, idx, logits, x, \
                                                       Wg, S, M, E, k, norm, chunk, dlogits, dx, dx_accumulate, partial)
    if (bf) { if (E <= 8) MOE_FUSED(true, 8, 4, 64); else MOE_FUSED(true, 16, 4, 128); }
    else { if (E <= 8) MOE_FUSED(false, 8, 4, 64); else MOE_FUSED(false, 16, 4, 128); }
#undef MOE_FUSED
    hipLaunchKernelGGL(gate_dwg_reduce, dim3((unsigned)((n + 63) / 64)), dim3(256), 0, st, partial, nchunk, M, E, dWg,
                       dgate_bias);
    return moe::check_launch();
  }
  hipLaunchKernelGGL(gate_dlogits, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, st, dw, w, idx, logits, S, E, k,
                     norm, dlogits);
  const dim3 grid_dx((unsigned)((M + WX_COLS - 1) / WX_COLS), (unsigned)((S + WX_TOK - 1) / WX_TOK));
  if (bf) hipLaunchKernelGGL(gate_dx_wide<true>, grid_dx, dim3(256), 0, st, dlogits, Wg, dx, S, M, E, dx_accumulate);
  else hipLaunchKernelGGL(gate_dx_wide<false>, grid_dx, dim3(256), 0, st, dlogits, Wg, dx, S, M, E, dx_accumulate);
  const int chunk = dwg_chunk(S, E);
  const int nchunk = (int)((S + chunk - 1) / chunk);
  float* partial = (float*)ws;
  const dim3 grid_w((unsigned)((M + 255) / 256), (unsigned)nchunk, (unsigned)((E + 63) / 64));
  if (bf) hipLaunchKernelGGL(gate_dwg_wide<true>, grid_w, dim3(256), 0, st, x, dlogits, partial, S, M, E, chunk);
  else hipLaunchKernelGGL(gate_dwg_wide<false>, grid_w, dim3(256), 0, st, x, dlogits, partial, S, M, E, chunk);
  hipLaunchKernelGGL(gate_dwg_reduce, dim3((unsigned)((n + 63) / 64)), dim3(256), 0, st, partial, nchunk, M, E, dWg,
                     dgate_bias);
  return moe::check_launch();
}
