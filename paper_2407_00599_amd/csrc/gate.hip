// Gate of the MoE layer (Section II-A "Gating Function") on the rank's MP token slice
// (Section III-B): logits = x Wg (+bias), top-k, combine weights, capacity slots.
//
// Kernels (wave64 throughout):
//   gate_logits_small_e : E <= 16.  One wave owns 64/EC tokens; lanes split M, so x is read
//                         once, coalesced, 16 B per lane; Wg goes through LDS as fp64, shared
//                         by the 8 waves of a block.  fp64 accumulation, then a halving
//                         cross-lane reduction that leaves lane i with output i.
//   gate_logits_mfma    : E > 16.  64 tokens x 64 experts per block on the fp64 matrix cores
//                         (v_mfma_f64_16x16x4_f64), K chunks converted to fp64 on their way into LDS.
//   gate_topk           : a group of W = pow2 >= E lanes per token; k rounds of an arg-max
//                         butterfly (ties -> lower expert index); softmax weights; per-block
//                         (choice, expert) histogram for the slot scan.
//   gate_scan           : one wave per expert; exclusive scan of the histograms over token blocks and
//                         over choices (choice-major priority), per-expert demand counts.
//   gate_slots          : rank of each (token, choice) inside its block via wave ballots,
//                         slot = base + rank if < C; inverse map; -1 tails of inv.
// The logits are accumulated in fp64 and rounded once to fp32, so the routing decision is
// taken on the same fp32 numbers a double-precision reference produces.
#include <mutex>
#include <type_traits>

#include "common.h"

// Scratch of moe_gate_topk_static: the per-block histograms and their scan, which moe_gate_topk keeps in
// the caller's workspace.  One copy per GPU, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels are given the address that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[MOE_GATE_STATIC_SCRATCH_BYTES];

namespace {

using namespace moe;

constexpr int GATE_TB = 64;   // tokens per block in gate_topk / gate_slots (one per thread)

template <bool BF16>
__device__ __forceinline__ void load8(const void* base, int64_t elem_off, bool ok, float* f) {
  if (!ok) {
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = 0.f;
    return;
  }
  if (BF16) {
    const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(base) + elem_off);
    unpack_bf16x8(v, f);
  } else {
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + elem_off);
    const float4 a = p[0], b = p[1];
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
}

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, mask, 64);
  hi = __shfl_xor(hi, mask, 64);
  return __hiloint2double(hi, lo);
}

// EC = experts held per lane (E <= EC), T tokens per wave, NW waves per block (T EC a power of two <= 64).
// The block walks M in chunks of 512.  Per chunk it converts Wg[chunk, :] to fp64 once into LDS (shared by
// the NW T tokens of the block, laid out [8][64 lanes][EC] so that a lane's EC doubles are contiguous),
// each lane takes 8 consecutive m of every one of its wave's T tokens
// (16-byte loads of x, the next chunk requested before this one is multiplied) and runs T*EC fp64 FMAs per
// m.  Blocks are small (4 waves, 4 or 2 tokens per wave) and light on registers so that several are
// resident per compute unit: one block's barriers and Wg staging hide behind another's FMAs.
template <int EC, bool BF16, int T, int NW>
__global__ __launch_bounds__(64 * NW, NW == 8 ? 4 : 1) void gate_logits_small_e(const void* __restrict__ x, const float* __restrict__ Wg,
                                                               const float* __restrict__ bias, float* __restrict__ logits,
                                                               int64_t S, int M, int E) {
  constexpr int NOUT = T * EC;
  static_assert(NOUT >= 2 && NOUT <= 64 && (NOUT & (NOUT - 1)) == 0, "T * EC must be a power of two <= 64");
  __shared__ double Ws[8 * 64 * EC];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t t0 = ((int64_t)blockIdx.x * NW + wave) * T;
  double acc[NOUT];
#pragma unroll
  for (int i = 0; i < NOUT; ++i) acc[i] = 0.0;

  typedef uint4 XRaw[BF16 ? 1 : 2];
  XRaw xr[T], xn[T];
  auto load_x = [&](XRaw* dst, int m0) {
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const bool ok = (t0 + t < S) && (m0 < M);
      const int64_t off = (t0 + t) * (int64_t)M + m0;
      if (BF16) {
        dst[t][0] = ok ? *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(x) + off) : make_uint4(0, 0, 0, 0);
      } else {
        const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(x) + off);
        dst[t][0] = ok ? p[0] : make_uint4(0, 0, 0, 0);
        dst[t][BF16 ? 0 : 1] = ok ? p[1] : make_uint4(0, 0, 0, 0);
      }
    }
  };
  load_x(xr, lane * 8);
  for (int mb = 0; mb < M; mb += 512) {
    __syncthreads();  // previous chunk's Ws fully consumed
    // slot i of the chunk, laid out [mm][expert pair][lane][2]: 16-byte reads at a 16-byte lane stride
    // slot i of the chunk holds expert i % EC of row m = 8 (i / EC % 64) + i / (64 EC): LDS writes are
    // contiguous (the Wg reads, 32-byte pieces, come from L2)
    for (int i = tid; i < 512 * EC; i += 64 * NW) {
      const int e = i % EC, lp = (i / EC) & 63, mm = i / (64 * EC);
      const int m = mb + lp * 8 + mm;
      Ws[i] = (double)((m < M && e < E) ? Wg[(int64_t)m * E + e] : 0.f);
    }
    __syncthreads();
    const bool more = mb + 512 < M;
    if (more) load_x(xn, mb + 512 + lane * 8);
#pragma unroll
    for (int mm = 0; mm < 8; ++mm) {
      double wd[EC];
#pragma unroll
      for (int e = 0; e < EC; ++e) wd[e] = Ws[(mm * 64 + lane) * EC + e];
#pragma unroll
      for (int t = 0; t < T; ++t) {
        float xf;
        if (BF16) {
          const uint32_t word = (&xr[t][0].x)[mm >> 1];
          xf = __uint_as_float((mm & 1) ? (word & 0xFFFF0000u) : (word << 16));
        } else {
          xf = __uint_as_float((&xr[t][mm >> 2].x)[mm & 3]);
        }
        const double xd = (double)xf;
#pragma unroll
        for (int e = 0; e < EC; ++e) acc[t * EC + e] = fma(xd, wd[e], acc[t * EC + e]);
      }
    }
    if (more) {
#pragma unroll
      for (int t = 0; t < T; ++t) {
        xr[t][0] = xn[t][0];
        if (!BF16) xr[t][BF16 ? 0 : 1] = xn[t][BF16 ? 0 : 1];
      }
    }
  }
  // halving reduction over the lanes: after the step with lane mask lm a lane whose bit lm is set holds
  // the upper half of its value list, summed with its partner's; once a single value is left the
  // remaining lane bits are plain butterfly sums.  At the end lane l holds value l >> log2(64 / NOUT).
#pragma unroll
  for (int st = 0; st < 6; ++st) {
    const int lm = 32 >> st;
    if ((NOUT >> st) > 1) {
      const int h = NOUT >> (st + 1);
      const bool up = (lane & lm) != 0;
#pragma unroll
      for (int i = 0; i < h; ++i) {
        const double keep = up ? acc[i + h] : acc[i];
        const double send = up ? acc[i] : acc[i + h];
        acc[i] = keep + shfl_xor_f64(send, lm);
      }
    } else {
      acc[0] += shfl_xor_f64(acc[0], lm);
    }
  }
  constexpr int REP = 64 / NOUT;          // lanes holding the same value
  const int o = lane / REP;
  const int t = o / EC, e = o % EC;
  if (lane % REP == 0 && t0 + t < S && e < E) {
    double v = acc[0];
    if (bias) v += (double)bias[e];
    logits[(t0 + t) * E + e] = (float)v;
  }
}

// E > 16: fp64 matrix cores.  v_mfma_f64_16x16x4_f64 multiplies a 16 x 4 by a 4 x 16 tile of doubles (lane l
// supplies A[l % 16][l / 16] and B[l / 16][l % 16], and receives D[4 r + l / 16][l % 16], r = 0..3).  A block of
// 4 waves owns 64 tokens x 64 experts (grid.y walks the expert blocks), a wave 16 tokens x 64 experts (four
// accumulator tiles).  M is walked in chunks of 32: x and Wg are converted to fp64 once on their way into LDS
// ([k][token] and [k][expert], pitch 80 doubles so that the two k planes of a 32-lane access fall into
// different banks), the next chunk's raw data being requested before the current one is multiplied.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
constexpr int LM_KC = 32, LM_PITCH = 80;
template <bool BF16>
__global__ __launch_bounds__(256) void gate_logits_mfma(const void* __restrict__ x, const float* __restrict__ Wg,
                                                        const float* __restrict__ bias, float* __restrict__ logits,
                                                        int64_t S, int M, int E) {
  __shared__ double xs[LM_KC * LM_PITCH];
  __shared__ double ws[LM_KC * LM_PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t tb = (int64_t)blockIdx.x * 64;
  const int e0 = blockIdx.y * 64;
  // staging roles: x -> token tid / 4, k offset 8 (tid % 4); Wg -> k row tid / 8, experts 8 (tid % 8)
  const int xt = tid >> 2, xk = (tid & 3) * 8;
  const int wk = tid >> 3, we = (tid & 7) * 8;
  uint4 xraw[BF16 ? 1 : 2];
  float4 wraw[2];
  auto fetch = [&](int k0) {
    const bool xok = (tb + xt < S) && (k0 + xk < M);     // M % 8 == 0: the 8 elements are in or out together
    const int64_t xo = (tb + xt) * (int64_t)M + k0 + xk;
    if (BF16) {
      xraw[0] = xok ? *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(x) + xo) : make_uint4(0, 0, 0, 0);
    } else {
      const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(x) + xo);
      xraw[0] = xok ? p[0] : make_uint4(0, 0, 0, 0);
      xraw[BF16 ? 0 : 1] = xok ? p[1] : make_uint4(0, 0, 0, 0);
    }
    const bool kok = k0 + wk < M;
    const float* wp = Wg + (int64_t)(k0 + wk) * E + e0 + we;
    float wv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) wv[u] = (kok && e0 + we + u < E) ? wp[u] : 0.f;   // E need not be a multiple of 4
    wraw[0] = make_float4(wv[0], wv[1], wv[2], wv[3]);
    wraw[1] = make_float4(wv[4], wv[5], wv[6], wv[7]);
  };
  auto stage = [&]() {
    float xf[8];
    if (BF16) {
      unpack_bf16x8(xraw[0], xf);
    } else {
      xf[0] = __uint_as_float(xraw[0].x); xf[1] = __uint_as_float(xraw[0].y); xf[2] = __uint_as_float(xraw[0].z);
      xf[3] = __uint_as_float(xraw[0].w); xf[4] = __uint_as_float(xraw[BF16 ? 0 : 1].x); xf[5] = __uint_as_float(xraw[BF16 ? 0 : 1].y);
      xf[6] = __uint_as_float(xraw[BF16 ? 0 : 1].z); xf[7] = __uint_as_float(xraw[BF16 ? 0 : 1].w);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) xs[(xk + u) * LM_PITCH + xt] = (double)xf[u];
    const float wv[8] = {wraw[0].x, wraw[0].y, wraw[0].z, wraw[0].w, wraw[1].x, wraw[1].y, wraw[1].z, wraw[1].w};
#pragma unroll
    for (int u = 0; u < 8; ++u) ws[wk * LM_PITCH + we + u] = (double)wv[u];
  };
  f64x4_t acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = f64x4_t{0.0, 0.0, 0.0, 0.0};

  fetch(0);
  for (int k0 = 0; k0 < M; k0 += LM_KC) {
    __syncthreads();   // the previous chunk is consumed
    stage();
    __syncthreads();
    if (k0 + LM_KC < M) fetch(k0 + LM_KC);
#pragma unroll
    for (int s4 = 0; s4 < LM_KC / 4; ++s4) {
      const int kr = (4 * s4 + (lane >> 4)) * LM_PITCH;
      const double a = xs[kr + wave * 16 + (lane & 15)];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const double bv = ws[kr + j * 16 + (lane & 15)];
        acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, bv, acc[j], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = e0 + j * 16 + (lane & 15);
    if (e >= E) continue;
    const double bj = bias ? (double)bias[e] : 0.0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int64_t t = tb + wave * 16 + 4 * r + (lane >> 4);
      if (t < S) logits[t * E + e] = (float)(acc[j][r] + bj);
    }
  }
}

// E <= 16 and many tokens: the fp64 matrix cores in their 4-block form.  v_mfma_f64_4x4x4_4b_f64 multiplies
// four independent 4 x 4 tiles by 4 x 4 tiles (k = 4) per instruction: lane l = 16 kk + 4 blk + i supplies
// A_blk[i][kk] and B_blk[kk][i], and receives D_blk[l / 16][l % 4] for blk = (l / 4) % 4 (layout confirmed with
// a one-wave probe).  On this chip the instruction runs on the fp64 vector units at their FMA rate (16
// cycles, during which the SIMD issues no other vector instruction), so what it buys is not arithmetic
// rate but structure: no cross-lane reduction, and every converted x value feeds 4 experts per
// instruction.  The conversion bf16 -> fp64 costs 20 cycles per 64 values (v_cvt_f64_f32 is quarter rate),
// as much as 1.25 matrix instructions, so each value is converted exactly once per wave: the four blocks are
// four token groups (16 tokens per instruction) and the experts are taken in NP passes of 4 that share the
// converted A operand (NP = 1, 2, 4 for E <= 4, 8, 16).
//   x:  fetched with whole-line requests (a lane takes 16 bytes, eight consecutive lanes one 128-byte piece
//       of a token row = 64 m, one instruction 8 rows) three steps ahead into registers, then passed through
//       a wave-private LDS region to reach the operand layout, in which neighbouring lanes hold DIFFERENT
//       tokens.  A lane of the operand layout reads 16 bytes = 8 consecutive m of its token, which feed 8
//       instructions per pass (the k index of instruction s is m = base + 8 kk + s: any bijection between
//       lanes and m serves, as long as A and B agree); a 64-m step is two such groups.  Row r stores piece p at
//       slot p ^ r, which makes both the row-wise writes and the operand-layout reads conflict-free.
//   Wg: converted to fp64 once per block and 512-m super-chunk on its way into LDS (double-buffered, one
//       barrier per super-chunk), in the order the lanes read it (16 bytes per lane; the four blocks read the
//       same addresses).
//   A block is TW x 2 waves: TW token waves (32 tokens each, two accumulator sets per pass), times 2 waves
//   that split the steps of a super-chunk and add their sums through LDS at the end.
//   Token rows and weights are fetched through buffer descriptors: an index outside the problem becomes an
//   out-of-range offset, which the hardware answers with zeros, so the loop body has no branches and the
//   compiler is free to interleave fetches, conversions and matrix instructions.
typedef unsigned int g4_u32x4_t __attribute__((ext_vector_type(4)));
constexpr uint32_t G4_OOB = 0xFFFFFFF0u;
constexpr int G4_KW = 2, G4_NS = 2, G4_SB = 4, G4_TS = 16;
constexpr int G4_SC = 64 * G4_SB * G4_KW;    // m per super-chunk
template <int NP, int TW>
__global__ __launch_bounds__(64 * TW * G4_KW) void gate_logits_mfma4(const bf16_t* __restrict__ x, const float* __restrict__ Wg,
                                                                      const float* __restrict__ bias, float* __restrict__ logits,
                                                                      int64_t S, int M, int E) {
  constexpr int KW = G4_KW, NS = G4_NS, SB = G4_SB, SC = G4_SC, TS = G4_TS;
  constexpr int NT = 64 * TW * KW;
  constexpr int ROWS = NS * TS;        // tokens per wave
  constexpr int NLD = ROWS / 8;        // fetches per step (8 rows each)
  constexpr int EP = 4 * NP;           // experts, padded
  constexpr int STEP_D = 64 * EP;      // doubles per 64-m step: [u 2][pass NP][p 4][kk 4][j 4][2]
  constexpr int BUF_D = SB * KW * STEP_D;
  constexpr int NST = SC * EP / NT;    // staged weights per thread and super-chunk
  static_assert(SC * EP % NT == 0, "staging layout");
  constexpr int RED_D = TW * KW * NS * NP * 64;
  __shared__ __attribute__((aligned(16))) double Bs[(2 * BUF_D > RED_D ? 2 * BUF_D : RED_D)];
  __shared__ __attribute__((aligned(16))) char Xs[TW * KW * ROWS * 128];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tw = wave / KW, kw = wave % KW;
  const int kk = lane >> 4, blk = (lane >> 2) & 3, li = lane & 3;
  const int tok_in_set = 4 * blk + li;
  const int64_t tset0 = ((int64_t)blockIdx.x * TW + tw) * ROWS;   // first token of this wave
  const int nsc = (M + SC - 1) / SC;

  // descriptors over the rank's token rows [S, M] and over Wg [M, E] (the host checks both are below 4 GiB)
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(x), 0, (uint32_t)((uint64_t)S * M * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Wg), 0, (uint32_t)((uint64_t)M * E * 4), 0x00020000);

  // ---- weights: global -> registers -> fp64 in LDS, in the lanes' read order ----
  // thread tid stages expert e = tid % EP of the rows ml0 + n (NT / EP), n = 0 .. NST - 1, of a super-chunk
  float wreg[NST];
  const int w_e = tid % EP, w_ml0 = tid / EP;
  const uint32_t w_step = (uint32_t)(NT / EP) * (uint32_t)E * 4u;
  auto fetch_w = [&](int sc) {
    const int m_first = sc * SC + w_ml0;
    const uint32_t base = ((uint32_t)m_first * (uint32_t)E + (uint32_t)w_e) * 4u;
#pragma unroll
    for (int n = 0; n < NST; ++n) {
      const bool ok = (m_first + n * (NT / EP) < M) & (w_e < E);
      const uint32_t off = ok ? base + (uint32_t)n * w_step : G4_OOB;
      wreg[n] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rw, (int)off, 0, 0));
    }
  };
  auto stage_w = [&](int buf) {
    double* dst = Bs + buf * BUF_D;
#pragma unroll
    for (int n = 0; n < NST; ++n) {
      const int idx = tid + n * NT, ml = idx / EP, e = idx % EP;
      const int st = ml >> 6, r = ml & 63, u = r >> 5, k4 = (r & 31) >> 3, sx = r & 7;   // group u = the 32-m half
      const int ps = e >> 2, j = e & 3;
      dst[st * STEP_D + ((((u * NP + ps) * 4 + (sx >> 1)) * 4 + k4) * 4 + j) * 2 + (sx & 1)] = (double)wreg[n];
    }
  };

  // ---- token rows: ring of SB register sets in the fetch layout (row = lane / 8, 16-byte piece = lane % 8) ----
  uint4 raw[SB][NLD];
  uint32_t row_off[NLD];                     // byte offset of this lane's piece at m = 0, or out of range
#pragma unroll
  for (int ld = 0; ld < NLD; ++ld) {
    const int64_t t = tset0 + 8 * ld + (lane >> 3);
    row_off[ld] = t < S ? (uint32_t)(((uint64_t)t * M + 8 * (lane & 7)) * 2) : G4_OOB;
  }
  auto fetch_x = [&](int n, int slot) {      // n = this wave's step number: super-chunk n / SB, step kw SB + n % SB
    const int m0 = (n / SB) * SC + (kw * SB + n % SB) * 64;
    const bool in = m0 + 8 * (lane & 7) < M;
#pragma unroll
    for (int ld = 0; ld < NLD; ++ld) {
      const uint32_t off = (row_off[ld] != G4_OOB && in) ? row_off[ld] + (uint32_t)m0 * 2u : G4_OOB;
      const g4_u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0);
      raw[slot][ld] = make_uint4(v.x, v.y, v.z, v.w);
    }
  };
  // wave-private LDS region [ROWS][8 pieces of 16 bytes], piece p of row r at slot p ^ (r % 8)
  char* xw = Xs + wave * (ROWS * 128);
  const int wr_off = (lane >> 3) * 128 + (((lane & 7) ^ (lane >> 3)) * 16);        // + ld * 1024
  int rd_off[NS][2];                                                              // set q, group u
#pragma unroll
  for (int q = 0; q < NS; ++q)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int r = q * TS + tok_in_set;
      rd_off[q][u] = r * 128 + (((4 * u + kk) ^ (r & 7)) * 16);
    }
  const int b_off = (kk * 4 + li) * 2;       // this lane's place among the 16 B lanes of a pass (doubles)

  double acc[NS][NP];
#pragma unroll
  for (int q = 0; q < NS; ++q)
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) acc[q][ps] = 0.0;

  fetch_w(0);
  const int nsteps = nsc * SB;
#pragma unroll
  for (int n = 0; n < SB - 1; ++n) fetch_x(n, n);
  stage_w(0);
  __syncthreads();

  for (int sc = 0; sc < nsc; ++sc) {
    if (sc + 1 < nsc) fetch_w(sc + 1);
    const double* bbuf = Bs + (sc & 1) * BUF_D + kw * SB * STEP_D + b_off;
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
      const int n = sc * SB + sb;
      if (n + SB - 1 < nsteps) fetch_x(n + SB - 1, (sb + SB - 1) % SB);
      // fetch layout -> operand layout through the wave's LDS region (LDS operations of a wave complete in order)
#pragma unroll
      for (int ld = 0; ld < NLD; ++ld) *reinterpret_cast<uint4*>(xw + ld * 1024 + wr_off) = raw[sb][ld];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        double da[NS][8];                    // the 8 values of this lane's piece, converted once
#pragma unroll
        for (int q = 0; q < NS; ++q) {
          const uint4 v = *reinterpret_cast<const uint4*>(xw + rd_off[q][u]);
#pragma unroll
          for (int sx = 0; sx < 8; ++sx) {
            const uint32_t wd = (&v.x)[sx >> 1];
            da[q][sx] = (double)__uint_as_float((sx & 1) ? (wd & 0xFFFF0000u) : (wd << 16));
          }
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          double2 b2[NP];
#pragma unroll
          for (int ps = 0; ps < NP; ++ps)
            b2[ps] = *reinterpret_cast<const double2*>(bbuf + sb * STEP_D + ((u * NP + ps) * 4 + p) * 32);
#pragma unroll
          for (int ps = 0; ps < NP; ++ps)
#pragma unroll
            for (int q = 0; q < NS; ++q) acc[q][ps] = __builtin_amdgcn_mfma_f64_4x4x4f64(da[q][2 * p], b2[ps].x, acc[q][ps], 0, 0, 0);
#pragma unroll
          for (int ps = 0; ps < NP; ++ps)
#pragma unroll
            for (int q = 0; q < NS; ++q) acc[q][ps] = __builtin_amdgcn_mfma_f64_4x4x4f64(da[q][2 * p + 1], b2[ps].y, acc[q][ps], 0, 0, 0);
        }
      }
    }
    if (sc + 1 < nsc) stage_w((sc + 1) & 1);
    __syncthreads();
  }

  // ---- add the KW partial sums through LDS (the weight buffers are free now) and store ----
  double* red = Bs;
  if (kw != 0) {
#pragma unroll
    for (int q = 0; q < NS; ++q)
#pragma unroll
      for (int ps = 0; ps < NP; ++ps) red[(((tw * KW + kw) * NS + q) * NP + ps) * 64 + lane] = acc[q][ps];
  }
  __syncthreads();
  if (kw == 0) {
    const int i = lane >> 4, j = lane & 3;
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      const int e = 4 * ps + j;
      const double bj = (bias != nullptr && e < E) ? (double)bias[e] : 0.0;
#pragma unroll
      for (int q = 0; q < NS; ++q) {
        double v = acc[q][ps];
#pragma unroll
        for (int w2 = 1; w2 < KW; ++w2) v += red[(((tw * KW + w2) * NS + q) * NP + ps) * 64 + lane];
        const int64_t t = tset0 + q * TS + 4 * blk + i;
        if (t < S && e < E) logits[t * E + e] = (float)(v + bj);
      }
    }
  }
}

struct Cand {
  float v;
  int e;  // INT_MAX = no candidate
};
__device__ __forceinline__ Cand better(Cand a, Cand b) {
  if (b.e == 0x7fffffff) return a;
  if (a.e == 0x7fffffff) return b;
  if (b.v > a.v || (b.v == a.v && b.e < a.e)) return b;
  return a;
}

// W lanes per token (W = pow2, W*EPL >= E).  Lane r of a group holds experts r, r+W, ...
// One block per GATE_TB tokens, min(W, 8) waves: the W passes (GATE_TB / W tokens each) are dealt to the waves.
template <int W, int EPL>
__global__ __launch_bounds__(GATE_TB * (W < 8 ? W : 8)) void gate_topk(const float* __restrict__ logits, int64_t S, int E, int k,
                                                      int norm_topk, int32_t* __restrict__ idx, float* __restrict__ w,
                                                      int32_t* __restrict__ blockhist) {
  __shared__ int hist[MOE_MAX_K * MOE_MAX_E];
  constexpr int NWV = W < 8 ? W : 8;   // waves per block
  constexpr int PPW = W / NWV;         // passes per wave
  const int tid = threadIdx.x & (GATE_TB - 1), wave = threadIdx.x / GATE_TB;
  for (int i = threadIdx.x; i < k * E; i += GATE_TB * NWV) hist[i] = 0;
  __syncthreads();
  const int r = tid % W;
  const int64_t tb0 = (int64_t)blockIdx.x * GATE_TB;
  constexpr int TPP = GATE_TB / W;  // tokens per pass
  constexpr int PG = PPW < 4 ? PPW : 4;  // passes whose logits are requested together
  float vv[PG][EPL];
  for (int pi = 0; pi < PPW; ++pi) {
    const int pass = wave * PPW + pi;
    if (pi % PG == 0) {
#pragma unroll
      for (int u = 0; u < PG; ++u) {
        const int64_t tu = tb0 + (pass + u) * TPP + tid / W;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          const int e = r + i * W;
          vv[u][i] = (tu < S && e < E) ? logits[tu * E + e] : 0.f;
        }
      }
    }
    const int64_t t = tb0 + pass * TPP + tid / W;
    const bool live = t < S;
    float v[EPL];
    unsigned taken = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const int e = r + i * W;
      float val = 0.f;
#pragma unroll
      for (int u = 0; u < PG; ++u)
        if (u == pi % PG) val = vv[u][i];
      v[i] = val;
      if (!(live && e < E)) taken |= 1u << i;
    }
    float selv[MOE_MAX_K];
    int sele[MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
      selv[j] = 0.f; sele[j] = 0;
      if (j < k) {
        Cand c{0.f, 0x7fffffff};
#pragma unroll
        for (int i = 0; i < EPL; ++i)
          if (!(taken & (1u << i))) c = better(c, Cand{v[i], r + i * W});
#pragma unroll
        for (int m = 1; m < W; m <<= 1) {
          Cand o;
          o.v = __shfl_xor(c.v, m, 64);
          o.e = __shfl_xor(c.e, m, 64);
          c = better(c, o);
        }
        selv[j] = c.v; sele[j] = c.e;
#pragma unroll
        for (int i = 0; i < EPL; ++i)
          if (c.e == r + i * W) taken |= 1u << i;
      }
    }
    // weights: exp(l - max) over the selected k, or over all experts
    const float mx = selv[0];
    float den = 0.f;
    if (norm_topk) {
#pragma unroll
      for (int j = 0; j < MOE_MAX_K; ++j)
        if (j < k) den += expf(selv[j] - mx);
    } else {
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        const int e = r + i * W;
        if (live && e < E) part += expf(v[i] - mx);
      }
#pragma unroll
      for (int m = 1; m < W; m <<= 1) part += __shfl_xor(part, m, 64);
      den = part;
    }
    if (live && r < k) {
      float lv = 0.f; int le = 0;
#pragma unroll
      for (int j = 0; j < MOE_MAX_K; ++j)
        if (j == r) { lv = selv[j]; le = sele[j]; }
      idx[t * k + r] = le;
      w[t * k + r] = expf(lv - mx) / den;
      atomicAdd(&hist[r * E + le], 1);
    }
  }
  __syncthreads();
  // stored [choice][expert][block] so the scan reads one (choice, expert) row contiguously
  for (int i = threadIdx.x; i < k * E; i += GATE_TB * NWV) blockhist[(int64_t)i * gridDim.x + blockIdx.x] = hist[i];
}

// blockhist[j][e][b] -> blockbase[j][e][b] = queue position of the first (token, choice j) of
// token block b at expert e.  Choice-major: all choice-0 demand of e precedes choice 1, ...
// One wave per expert; 64 blocks are scanned per step with a shuffle prefix sum.
__global__ __launch_bounds__(256) void gate_scan(const int32_t* __restrict__ blockhist, int nblk, int E, int k,
                                                 int32_t* __restrict__ blockbase, int32_t* __restrict__ counts) {
  const int lane = threadIdx.x & 63;
  const int e = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (e >= E) return;
  int run = 0;
  for (int j = 0; j < k; ++j) {
    const int64_t row = ((int64_t)j * E + e) * nblk;
    for (int b0 = 0; b0 < nblk; b0 += 64) {
      const int b = b0 + lane;
      const int h = b < nblk ? blockhist[row + b] : 0;
      int incl = h;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
      }
      if (b < nblk) blockbase[row + b] = run + incl - h;
      run += __shfl(incl, 63, 64);
    }
  }
  if (lane == 0) counts[e] = run;
}

// SCAN = false: queue positions of the block's first tokens come from gate_scan (blockbase, counts).
// SCAN = true (few token blocks): every block works them out itself from the per-block histograms --
// for each (choice j, expert e) the demand of the earlier blocks, plus all demand of the earlier
// choices -- which saves the scan launch; block 0 also writes counts.  Same integers either way.
template <bool SCAN>
__global__ __launch_bounds__(GATE_TB) void gate_slots(const int32_t* __restrict__ idx, const int32_t* __restrict__ blockbase,
                                                       int32_t* __restrict__ counts, int64_t S, int E, int k,
                                                       int64_t C, int32_t* __restrict__ slot, int32_t* __restrict__ inv) {
  static_assert(GATE_TB == 64, "one wave per block");
  __shared__ int wavecnt[GATE_TB / 64][MOE_MAX_E];
  __shared__ int base_s[SCAN ? MOE_MAX_K * MOE_MAX_E : 1];   // queue position of this block's first (j, e) token
  __shared__ int tot_s[SCAN ? MOE_MAX_K * MOE_MAX_E : 1];    // demand of (j, e) over all blocks
  __shared__ int count_s[SCAN ? MOE_MAX_E : 1];              // total demand of expert e
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t t = (int64_t)blockIdx.x * GATE_TB + tid;
  const bool live = t < S;
  if (SCAN) {
    // here blockbase holds the histograms [j][e][b].  Lanes run over b; sixteen (j, e) rows at a time, so that
    // sixteen loads are in flight per lane; the wave-wide sums of a row: its total and the part of the
    // blocks before this one.
    const int nblk = (int)gridDim.x, me = (int)blockIdx.x, npair = k * E;
    for (int p0 = 0; p0 < npair; p0 += 16) {
      int tot[16], pre[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) tot[u] = pre[u] = 0;
      for (int b0 = 0; b0 < nblk; b0 += 64) {
        const int b = b0 + lane;
        int h[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) h[u] = (b < nblk && p0 + u < npair) ? blockbase[(int64_t)(p0 + u) * nblk + b] : 0;
#pragma unroll
        for (int u = 0; u < 16; ++u) { tot[u] += h[u]; pre[u] += b < me ? h[u] : 0; }
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) { tot[u] += __shfl_xor(tot[u], o, 64); pre[u] += __shfl_xor(pre[u], o, 64); }
        if (lane == 0 && p0 + u < npair) { base_s[p0 + u] = pre[u]; tot_s[p0 + u] = tot[u]; }
      }
    }
    __syncthreads();
    // choice-major queues: all demand of the earlier choices at expert e comes first
    for (int e = tid; e < E; e += GATE_TB) {
      int run = 0;
      for (int j = 0; j < k; ++j) {
        const int i = j * E + e;
        base_s[i] += run;
        run += tot_s[i];
      }
      count_s[e] = run;
      if (me == 0) counts[e] = run;
    }
    __syncthreads();
  }
  for (int j = 0; j < k; ++j) {
    for (int i = tid; i < (GATE_TB / 64) * MOE_MAX_E; i += GATE_TB) (&wavecnt[0][0])[i] = 0;
    __syncthreads();
    const int e = live ? idx[t * k + j] : -1;
    int rank = 0;
    unsigned long long todo = __ballot(live);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int e0 = __shfl(e, leader, 64);
      const unsigned long long same = __ballot(live && e == e0);
      if (e == e0) {
        rank = __popcll(same & ((1ull << lane) - 1ull));
        if (lane == leader) wavecnt[wv][e0] = __popcll(same);
      }
      todo &= ~same;
    }
    __syncthreads();
    if (live) {
      int pos = (SCAN ? base_s[j * E + e] : blockbase[((int64_t)j * E + e) * gridDim.x + blockIdx.x]) + rank;
      for (int q = 0; q < wv; ++q) pos += wavecnt[q][e];
      const bool keep = pos < C;
      slot[t * k + j] = keep ? pos : -1;
      if (keep) inv[(int64_t)e * C + pos] = (int32_t)(t * k + j);
    }
    __syncthreads();
  }
  // empty tail of every expert's block: slots [min(counts[e], C), C)
  const int64_t total = (int64_t)E * C;
  for (int64_t i = (int64_t)blockIdx.x * GATE_TB + tid; i < total; i += (int64_t)gridDim.x * GATE_TB) {
    const int e = (int)(i / C);
    const int64_t c = i - (int64_t)e * C;
    if (c >= (SCAN ? count_s[e] : counts[e])) inv[i] = -1;
  }
}

template <int W, int EPL>
void launch_topk(const float* logits, int64_t S, int E, int k, int norm, int32_t* idx, float* w, int32_t* bh,
                 int nblk, hipStream_t st) {
  hipLaunchKernelGGL((gate_topk<W, EPL>), dim3(nblk), dim3(GATE_TB * (W < 8 ? W : 8)), 0, st, logits, S, E, k, norm,
                     idx, w, bh);
}

}  // namespace

// Address of the current device's copy of the scratch array, looked up once per device (with that device
// current) and kept; nullptr if the runtime refuses.
static void* static_scratch() {
  constexpr int MAX_DEV = 64;
  static void* ptr[MAX_DEV] = {};
  static std::mutex mu;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    ptr[dev] = p;
  }
  return ptr[dev];
}

extern "C" size_t moe_gate_workspace_bytes(int64_t S, int E, int k) {
  if (S < 1 || E < 1 || k < 1) return 0;
  const int64_t nblk = (S + GATE_TB - 1) / GATE_TB;
  return moe::align_up((size_t)nblk * k * E * sizeof(int32_t), 256) * 2;
}

// ws == nullptr: the workspace is this GPU's static scratch array (moe_gate_topk_static)
static int gate_topk_impl(const void* x, int x_dtype, const float* Wg, const float* gate_bias,
                          int64_t S_total, int M, int E, int k, int64_t C, int mp_idx, int n_mp, int norm_topk,
                          float* logits, int32_t* idx, int32_t* slot, float* w, int32_t* inv, int32_t* counts,
                          void* ws, size_t ws_bytes, bool static_ws, void* stream) {
  MOE_REQUIRE(n_mp >= 1 && mp_idx >= 0 && mp_idx < n_mp, MOE_EINVAL);
  MOE_REQUIRE(S_total >= 1 && S_total % n_mp == 0, MOE_EINVAL);
  const int64_t S = S_total / n_mp;
  if (int rc = moe::common_shape_check(S, x ? M : 8, E, k, C)) return rc;
  MOE_REQUIRE(norm_topk >= -1 && norm_topk <= 1, MOE_EINVAL);
  if (x) {
    MOE_REQUIRE(x_dtype == MOE_F32 || x_dtype == MOE_BF16, MOE_EINVAL);
    MOE_REQUIRE_PTR(x);
    MOE_REQUIRE_PTR(Wg);
  }
  MOE_OPTIONAL_PTR(gate_bias);
  MOE_REQUIRE_PTR(logits); MOE_REQUIRE_PTR(idx); MOE_REQUIRE_PTR(slot); MOE_REQUIRE_PTR(w);
  MOE_REQUIRE_PTR(inv); MOE_REQUIRE_PTR(counts);
  const size_t need = moe_gate_workspace_bytes(S, E, k);
  if (static_ws) {
    MOE_REQUIRE(need <= MOE_GATE_STATIC_SCRATCH_BYTES, MOE_ESCRATCH);
    ws = static_scratch();
    MOE_REQUIRE(ws != nullptr, MOE_ELAUNCH);
  } else {
    MOE_REQUIRE(ws != nullptr && ws_bytes >= need, MOE_EWORKSPACE);
    MOE_REQUIRE(moe::aligned16(ws), MOE_EALIGN);
  }
  const int norm = norm_topk < 0 ? (k >= 2 ? 1 : 0) : norm_topk;
  hipStream_t st = (hipStream_t)stream;
  const int nblk = (int)((S + GATE_TB - 1) / GATE_TB);
  int32_t* blockhist = (int32_t*)ws;
  int32_t* blockbase = (int32_t*)((char*)ws + need / 2);

  if (x) {
    const bool bf = x_dtype == MOE_BF16;
    const size_t esz = bf ? 2 : 4;
    const void* xs = (const char*)x + (size_t)mp_idx * S * M * esz;
    if (E <= 16 && bf && S >= 8192 && (uint64_t)S * (uint64_t)M * 2 <= 0xFFFFFFF0ull) {
      // fp64 matrix cores; TW token waves (32 tokens each) per block so that the grid has about two blocks per
      // compute unit or more
      const int tw = S >= 512 * 4 * 32 ? 4 : S >= 512 * 2 * 32 ? 2 : 1;
      const int64_t tpb = (int64_t)tw * G4_NS * G4_TS;     // tokens per block
      const dim3 grid((unsigned)((S + tpb - 1) / tpb)), block(64 * tw * G4_KW);
      const bf16_t* xb = (const bf16_t*)xs;
#define LAUNCH_M4(np, tw_) hipLaunchKernelGGL((gate_logits_mfma4<np, tw_>), grid, block, 0, st, xb, Wg, gate_bias, logits, S, M, E)
#define LAUNCH_M4_TW(np) do { if (tw == 4) LAUNCH_M4(np, 4); else if (tw == 2) LAUNCH_M4(np, 2); else LAUNCH_M4(np, 1); } while (0)
      if (E <= 4) LAUNCH_M4_TW(1); else if (E <= 8) LAUNCH_M4_TW(2); else LAUNCH_M4_TW(4);
#undef LAUNCH_M4_TW
#undef LAUNCH_M4
    } else if (E <= 16) {
      const int EC = E <= 8 ? 8 : 16;
      const int T = E <= 8 ? 4 : 2;
      // many tokens: 8-wave blocks halve the Wg staging work per token; few tokens: 4-wave blocks fill the chip
      const int nw = (S >= 16384 && bf) ? 8 : 4;
      const dim3 grid((unsigned)((S + nw * T - 1) / (nw * T))), block(64 * nw);
#define LAUNCH_SMALL(ec, t) do { \
    if (bf && nw == 8) hipLaunchKernelGGL((gate_logits_small_e<ec, true, t, 8>), grid, block, 0, st, xs, Wg, gate_bias, logits, S, M, E); \
    else if (bf) hipLaunchKernelGGL((gate_logits_small_e<ec, true, t, 4>), grid, block, 0, st, xs, Wg, gate_bias, logits, S, M, E); \
    else hipLaunchKernelGGL((gate_logits_small_e<ec, false, t, 4>), grid, block, 0, st, xs, Wg, gate_bias, logits, S, M, E); } while (0)
      if (EC == 8) LAUNCH_SMALL(8, 4); else LAUNCH_SMALL(16, 2);
#undef LAUNCH_SMALL
    } else {
      const dim3 grid((unsigned)((S + 63) / 64), (unsigned)((E + 63) / 64)), block(256);
      if (bf) hipLaunchKernelGGL((gate_logits_mfma<true>), grid, block, 0, st, xs, Wg, gate_bias, logits, S, M, E);
      else hipLaunchKernelGGL((gate_logits_mfma<false>), grid, block, 0, st, xs, Wg, gate_bias, logits, S, M, E);
    }
  }
  if (E <= 1) launch_topk<1, 1>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else if (E <= 2) launch_topk<2, 1>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else if (E <= 4) launch_topk<4, 1>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else if (E <= 8) launch_topk<8, 1>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else if (E <= 16) launch_topk<16, 1>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else if (E <= 32) launch_topk<32, 1>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else if (E <= 64) launch_topk<64, 1>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else if (E <= 128) launch_topk<64, 2>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  else launch_topk<64, 4>(logits, S, E, k, norm, idx, w, blockhist, nblk, st);
  if ((int64_t)nblk * k * E <= 16384) {   // every block reads all histograms itself: at most 64 KiB each
    hipLaunchKernelGGL(gate_slots<true>, dim3(nblk), dim3(GATE_TB), 0, st, idx, blockhist, counts, S, E, k, C, slot, inv);
  } else {
    hipLaunchKernelGGL(gate_scan, dim3((E + 3) / 4), dim3(256), 0, st, blockhist, nblk, E, k, blockbase, counts);
    hipLaunchKernelGGL(gate_slots<false>, dim3(nblk), dim3(GATE_TB), 0, st, idx, blockbase, counts, S, E, k, C, slot, inv);
  }
  return moe::check_launch();
}

extern "C" int moe_gate_topk(const void* x, int x_dtype, const float* Wg, const float* gate_bias,
                             int64_t S_total, int M, int E, int k, int64_t C, int mp_idx, int n_mp, int norm_topk,
                             float* logits, int32_t* idx, int32_t* slot, float* w, int32_t* inv, int32_t* counts,
                             void* ws, size_t ws_bytes, void* stream) {
  return gate_topk_impl(x, x_dtype, Wg, gate_bias, S_total, M, E, k, C, mp_idx, n_mp, norm_topk, logits, idx, slot, w,
                        inv, counts, ws, ws_bytes, false, stream);
}

extern "C" int moe_gate_topk_static(const void* x, int x_dtype, const float* Wg, const float* gate_bias,
                                    int64_t S_total, int M, int E, int k, int64_t C, int mp_idx, int n_mp,
                                    int norm_topk, float* logits, int32_t* idx, int32_t* slot, float* w,
                                    int32_t* inv, int32_t* counts, void* stream) {
  return gate_topk_impl(x, x_dtype, Wg, gate_bias, S_total, M, E, k, C, mp_idx, n_mp, norm_topk, logits, idx, slot, w,
                        inv, counts, nullptr, 0, true, stream);
}
