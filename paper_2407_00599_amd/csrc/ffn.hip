// Expert FFN of one ESP shard, forward and backward (Section II-A "Experts": weights (M,H) and
// (H,M) around an activation; hidden dimension sharded as Y = sum_p W2^(p) f(W1^(p) X),
// Section II-B, which ESP applies to experts).
//
// Six grouped GEMMs (one group per local expert g, all experts in one launch):
//   forward   Z  = X  * W1[:, h0:h0+H_l]        kind NN   epilogue: store Z and Act = GeLU(Z)
//             Y  = Act * W2[h0:h0+H_l, :]       kind NN
//   backward  dA = dY * W2[h0:h0+H_l, :]^T      kind NT   epilogue: dZ = dA * GeLU'(Z), Act = GeLU(Z)
//             dW2[h0:h0+H_l, :] = Act^T * dY    kind TN   (reduction over the expert's n_src*C rows)
//             dW1[:, h0:h0+H_l] = X^T * dZ      kind TN
//             dX = dZ * W1[:, h0:h0+H_l]^T      kind NT
//
// Activation-type operands live in the AlltoAll receive layout [n_src, G, C, ld]: the rows of
// expert g are n_src separate chunks of C rows.  The kernels address "virtual row" r of expert
// g at physical row ((r / C) * G + g) * C + r % C, so no permutation pass is needed and only
// the last row tile of an expert is ragged.
//
// bf16 path: MFMA v_mfma_f32_32x32x16_bf16, fp32 accumulation.  Both MFMA operands want 8
// consecutive k per lane, so LDS tiles are always [row][k] with k contiguous (row pitch 64+8
// bf16, which makes the 16-byte fragment reads bank-conflict free).  Operands whose memory
// layout has k as the slow index (W1/W2 in the NN GEMMs, both operands of the TN GEMMs) are
// transposed in registers (8x8 blocks, v_perm) on their way from global memory to LDS.
// Global->register loads of tile kt+1 are issued before the MFMAs of tile kt (LDS double
// buffer, one barrier per k tile).  The MFMA is issued with the operands swapped (D^T = B^T
// A^T) so that a lane ends up with 4 consecutive output columns and stores 8 bytes.
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs) works
// on one contiguous range of tiles and its L2 sees the same weight panels.
//
// fp32 path: a plain LDS-tiled kernel with fp64 accumulation, for the small fp32 configuration.
#include "common.h"

namespace {

using namespace moe;

enum { KIND_NN = 1, KIND_NT = 2, KIND_TN = 3 };
enum { EPI_STORE = 0, EPI_GELU = 1, EPI_DGELU = 2 };

struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  void* C2;         // second output (Act) for EPI_GELU / EPI_DGELU
  const void* Zin;  // saved pre-activation for EPI_DGELU
  int G, n_src;
  int Cc;           // rows per chunk (capacity C)
  int R;            // n_src * Cc: virtual rows per expert
  int Mdim, Ndim, Kdim;
  int64_t lda, ldb, ldc;             // leading dimensions, elements
  int64_t b_goff, c_goff;            // per-expert stride of weight-type operands, elements
  int64_t b_off, c_off;              // constant offset of the ESP slice, elements
  int tiles_m, tiles_n, total_tiles;
  int kchunks;                       // TN: k tiles per chunk = ceil(Cc / 64)
};

__device__ __forceinline__ int64_t phys_row(int r, int g, int G, int Cc) {
  const int s = r / Cc;
  return ((int64_t)s * G + g) * Cc + (r - s * Cc);
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int KT = 64;          // k tile
constexpr int PITCH = KT + 8;   // LDS row pitch in bf16 elements (144 bytes)

// 8x8 transpose of 16-bit elements: in[i] holds 8 consecutive n for k = i; out[n] holds 8
// consecutive k for that n.
__device__ __forceinline__ void transpose8x8(const uint4* in, uint4* out) {
  const uint32_t* I = reinterpret_cast<const uint32_t*>(in);
  uint32_t* O = reinterpret_cast<uint32_t*>(out);
#pragma unroll
  for (int n = 0; n < 8; ++n) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t a = I[(2 * d) * 4 + n / 2];      // k = 2d
      const uint32_t b = I[(2 * d + 1) * 4 + n / 2];  // k = 2d+1
      O[n * 4 + d] = (n & 1) ? __builtin_amdgcn_perm(b, a, 0x07060302u) : __builtin_amdgcn_perm(b, a, 0x05040100u);
    }
  }
}

// 4(k) x 8(n) -> 8 rows of 4 consecutive k (8 bytes each)
__device__ __forceinline__ void transpose4x8(const uint4* in, uint2* out) {
  const uint32_t* I = reinterpret_cast<const uint32_t*>(in);
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    const uint32_t a0 = I[0 * 4 + n / 2], b0 = I[1 * 4 + n / 2];
    const uint32_t a1 = I[2 * 4 + n / 2], b1 = I[3 * 4 + n / 2];
    if (n & 1) {
      out[n].x = __builtin_amdgcn_perm(b0, a0, 0x07060302u);
      out[n].y = __builtin_amdgcn_perm(b1, a1, 0x07060302u);
    } else {
      out[n].x = __builtin_amdgcn_perm(b0, a0, 0x05040100u);
      out[n].y = __builtin_amdgcn_perm(b1, a1, 0x05040100u);
    }
  }
}

// Staging of one operand tile [ROWS x KT] (rows = output-dim index, k contiguous in LDS).
// DIRECT: memory has k contiguous.  Thread handles chunks c = tid + i*NT, row = c/8, kc = c%8.
// TRANSPOSED: memory has the row index contiguous and k as the slow index.  Thread handles
// 8(k) x 8(row) blocks (or 4 x 8 half blocks when there are fewer blocks than threads).
template <int ROWS, int NT>
struct Stage {
  static constexpr int NCH = ROWS * 8 / NT;            // direct: 16-byte chunks per thread
  static constexpr int NBLK = ROWS;                    // transposed: number of 8x8 blocks (ROWS/8 * 8)
  static constexpr bool HALF = NBLK < NT;              // 4x8 half blocks
  static constexpr int NB = HALF ? 1 : NBLK / NT;      // blocks per thread
  static_assert(NCH >= 1 && (HALF ? NBLK * 2 == NT : NBLK % NT == 0), "tile/thread mismatch");
  uint4 reg[NCH];                                      // NCH == 8*NB (full) or 4 (half)
};

template <int TM, int TN, int WM, int WN, int KIND, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void ffn_gemm_bf16(const GemmArgs p) {
  constexpr int NT = WM * WN * 64;
  constexpr int TMW = TM / WM, TNW = TN / WN;  // per-wave tile
  constexpr int MB = TMW / 32, NBK = TNW / 32;
  constexpr bool A_TR = (KIND == KIND_TN);
  constexpr bool B_TR = (KIND == KIND_NN || KIND == KIND_TN);
  using SA = Stage<TM, NT>;
  using SB = Stage<TN, NT>;

  __shared__ __attribute__((aligned(16))) bf16_t smem[2 * (TM + TN) * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- tile assignment (XCD-contiguous remap) ----
  const int per_xcd = (p.total_tiles + 7) / 8;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile >= p.total_tiles) return;
  const int tiles_per_g = p.tiles_m * p.tiles_n;
  const int g = tile / tiles_per_g;
  const int tr = tile - g * tiles_per_g;
  const int tm = tr / p.tiles_n, tn = tr - tm * p.tiles_n;
  const int m0 = tm * TM, n0 = tn * TN;

  const bf16_t* __restrict__ Ab = reinterpret_cast<const bf16_t*>(p.A);
  const bf16_t* __restrict__ Bb = reinterpret_cast<const bf16_t*>(p.B);

  // ---- per-thread staging coordinates ----
  // direct: row = tid/8 + i*(NT/8), kc = tid%8
  // transposed: full blocks: kb = bi%8, r8 = bi/8 (bi = tid + i*NT); half: kb4 = tid%16, r8 = tid/16
  int64_t a_rowoff[SA::NCH];  // direct A: element offset of the row start, -1 = out of range
  (void)a_rowoff;
  if (!A_TR) {
#pragma unroll
    for (int i = 0; i < SA::NCH; ++i) {
      const int r = m0 + (tid >> 3) + i * (NT / 8);
      a_rowoff[i] = (r < p.Mdim) ? phys_row(r, g, p.G, p.Cc) * p.lda : -1;
    }
  }
  const int64_t b_base = (int64_t)g * p.b_goff + p.b_off;

  const int nk = (KIND == KIND_TN) ? p.n_src * p.kchunks : (p.Kdim + KT - 1) / KT;

  SA sa;
  SB sb;

  auto load_tiles = [&](int kt) {
    // ---------------- A ----------------
    if (!A_TR) {
      const int k = kt * KT + (tid & 7) * 8;
#pragma unroll
      for (int i = 0; i < SA::NCH; ++i) {
        const bool ok = a_rowoff[i] >= 0 && k < p.Kdim;
        sa.reg[i] = ok ? *reinterpret_cast<const uint4*>(Ab + a_rowoff[i] + k) : make_uint4(0, 0, 0, 0);
      }
    } else {
      const int s = kt / p.kchunks;
      const int c0 = (kt - s * p.kchunks) * KT;
      const int64_t chunk_row = ((int64_t)s * p.G + g) * p.Cc;
      if (!SA::HALF) {
#pragma unroll
        for (int b = 0; b < SA::NB; ++b) {
          const int bi = tid + b * NT;
          const int kb = bi & 7, r8 = bi >> 3;
          const int col = m0 + r8 * 8;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int c = c0 + kb * 8 + i;
            const bool ok = c < p.Cc && col < p.Mdim;
            sa.reg[b * 8 + i] = ok ? *reinterpret_cast<const uint4*>(Ab + (chunk_row + c) * p.lda + col)
                                   : make_uint4(0, 0, 0, 0);
          }
        }
      } else {
        const int kb4 = tid & 15, r8 = tid >> 4;
        const int col = m0 + r8 * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int c = c0 + kb4 * 4 + i;
          const bool ok = c < p.Cc && col < p.Mdim;
          sa.reg[i] = ok ? *reinterpret_cast<const uint4*>(Ab + (chunk_row + c) * p.lda + col)
                         : make_uint4(0, 0, 0, 0);
        }
      }
    }
    // ---------------- B ----------------
    if (!B_TR) {  // NT: weight rows n, k contiguous
      const int k = kt * KT + (tid & 7) * 8;
#pragma unroll
      for (int i = 0; i < SB::NCH; ++i) {
        const int n = n0 + (tid >> 3) + i * (NT / 8);
        const bool ok = n < p.Ndim && k < p.Kdim;
        sb.reg[i] = ok ? *reinterpret_cast<const uint4*>(Bb + b_base + (int64_t)n * p.ldb + k) : make_uint4(0, 0, 0, 0);
      }
    } else {
      int64_t krow0;  // element offset of k row 0 of this tile
      int klim;       // number of valid k rows in this tile
      if (KIND == KIND_NN) {
        krow0 = b_base + (int64_t)kt * KT * p.ldb;
        klim = p.Kdim - kt * KT;
      } else {
        const int s = kt / p.kchunks;
        const int c0 = (kt - s * p.kchunks) * KT;
        krow0 = (((int64_t)s * p.G + g) * p.Cc + c0) * p.ldb;
        klim = p.Cc - c0;
      }
      if (!SB::HALF) {
#pragma unroll
        for (int b = 0; b < SB::NB; ++b) {
          const int bi = tid + b * NT;
          const int kb = bi & 7, r8 = bi >> 3;
          const int col = n0 + r8 * 8;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int kk = kb * 8 + i;
            const bool ok = kk < klim && col < p.Ndim;
            sb.reg[b * 8 + i] = ok ? *reinterpret_cast<const uint4*>(Bb + krow0 + (int64_t)kk * p.ldb + col)
                                   : make_uint4(0, 0, 0, 0);
          }
        }
      } else {
        const int kb4 = tid & 15, r8 = tid >> 4;
        const int col = n0 + r8 * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int kk = kb4 * 4 + i;
          const bool ok = kk < klim && col < p.Ndim;
          sb.reg[i] = ok ? *reinterpret_cast<const uint4*>(Bb + krow0 + (int64_t)kk * p.ldb + col)
                         : make_uint4(0, 0, 0, 0);
        }
      }
    }
  };

  auto store_tiles = [&](int buf) {
    bf16_t* As = smem + buf * (TM + TN) * PITCH;
    bf16_t* Bs = As + TM * PITCH;
    if (!A_TR) {
#pragma unroll
      for (int i = 0; i < SA::NCH; ++i) {
        const int row = (tid >> 3) + i * (NT / 8);
        *reinterpret_cast<uint4*>(As + row * PITCH + (tid & 7) * 8) = sa.reg[i];
      }
    } else if (!SA::HALF) {
#pragma unroll
      for (int b = 0; b < SA::NB; ++b) {
        const int bi = tid + b * NT;
        const int kb = bi & 7, r8 = bi >> 3;
        uint4 t[8];
        transpose8x8(&sa.reg[b * 8], t);
#pragma unroll
        for (int n = 0; n < 8; ++n) *reinterpret_cast<uint4*>(As + (r8 * 8 + n) * PITCH + kb * 8) = t[n];
      }
    } else {
      const int kb4 = tid & 15, r8 = tid >> 4;
      uint2 t[8];
      transpose4x8(sa.reg, t);
#pragma unroll
      for (int n = 0; n < 8; ++n) *reinterpret_cast<uint2*>(As + (r8 * 8 + n) * PITCH + kb4 * 4) = t[n];
    }
    if (!B_TR) {
#pragma unroll
      for (int i = 0; i < SB::NCH; ++i) {
        const int row = (tid >> 3) + i * (NT / 8);
        *reinterpret_cast<uint4*>(Bs + row * PITCH + (tid & 7) * 8) = sb.reg[i];
      }
    } else if (!SB::HALF) {
#pragma unroll
      for (int b = 0; b < SB::NB; ++b) {
        const int bi = tid + b * NT;
        const int kb = bi & 7, r8 = bi >> 3;
        uint4 t[8];
        transpose8x8(&sb.reg[b * 8], t);
#pragma unroll
        for (int n = 0; n < 8; ++n) *reinterpret_cast<uint4*>(Bs + (r8 * 8 + n) * PITCH + kb * 8) = t[n];
      }
    } else {
      const int kb4 = tid & 15, r8 = tid >> 4;
      uint2 t[8];
      transpose4x8(sb.reg, t);
#pragma unroll
      for (int n = 0; n < 8; ++n) *reinterpret_cast<uint2*>(Bs + (r8 * 8 + n) * PITCH + kb4 * 4) = t[n];
    }
  };

  f32x16_t acc[MB][NBK];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NBK; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  load_tiles(0);
  store_tiles(0);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_tiles(kt + 1);
    const bf16_t* As = smem + buf * (TM + TN) * PITCH + (wm * TMW + (lane & 31)) * PITCH + (lane >> 5) * 8;
    const bf16_t* Bs = smem + buf * (TM + TN) * PITCH + TM * PITCH + (wn * TNW + (lane & 31)) * PITCH + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
      bf16x8_t af[MB], bfr[NBK];
#pragma unroll
      for (int i = 0; i < MB; ++i) af[i] = *reinterpret_cast<const bf16x8_t*>(As + i * 32 * PITCH + kk * 16);
#pragma unroll
      for (int j = 0; j < NBK; ++j) bfr[j] = *reinterpret_cast<const bf16x8_t*>(Bs + j * 32 * PITCH + kk * 16);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NBK; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds output row m = .. + lane%32 and, for q = 0..15,
  //      column n = .. + 8*(q/4) + 4*(lane/32) + q%4 ----
  bf16_t* __restrict__ Cb = reinterpret_cast<bf16_t*>(p.C);
  bf16_t* __restrict__ C2b = reinterpret_cast<bf16_t*>(p.C2);
  const bf16_t* __restrict__ Zb = reinterpret_cast<const bf16_t*>(p.Zin);
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    const int m = m0 + wm * TMW + i * 32 + (lane & 31);
    if (m >= p.Mdim) continue;
    int64_t crow;
    if (KIND == KIND_TN) crow = (int64_t)g * p.c_goff + p.c_off + (int64_t)m * p.ldc;
    else crow = phys_row(m, g, p.G, p.Cc) * p.ldc;
#pragma unroll
    for (int j = 0; j < NBK; ++j) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int n = n0 + wn * TNW + j * 32 + q4 * 8 + (lane >> 5) * 4;
        if (n >= p.Ndim) continue;
        float v[4] = {acc[i][j][q4 * 4 + 0], acc[i][j][q4 * 4 + 1], acc[i][j][q4 * 4 + 2], acc[i][j][q4 * 4 + 3]};
        if (EPI == EPI_STORE) {
          *reinterpret_cast<uint2*>(Cb + crow + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        } else if (EPI == EPI_GELU) {
          *reinterpret_cast<uint2*>(Cb + crow + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          float a[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) a[e] = gelu_f(v[e]);
          *reinterpret_cast<uint2*>(C2b + crow + n) = make_uint2(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]));
        } else {
          const uint2 zq = *reinterpret_cast<const uint2*>(Zb + crow + n);
          const float z[4] = {__uint_as_float(zq.x << 16), __uint_as_float(zq.x & 0xFFFF0000u),
                              __uint_as_float(zq.y << 16), __uint_as_float(zq.y & 0xFFFF0000u)};
          float a[4], d[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float ge, dg;
            gelu_and_grad(z[e], ge, dg);
            a[e] = ge;
            d[e] = v[e] * dg;
          }
          *reinterpret_cast<uint2*>(Cb + crow + n) = make_uint2(pack_bf16x2(d[0], d[1]), pack_bf16x2(d[2], d[3]));
          *reinterpret_cast<uint2*>(C2b + crow + n) = make_uint2(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]));
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// fp32 kernel: 64x64 tile, 256 threads, 4x4 outputs per thread, fp64 accumulation.
// ------------------------------------------------------------------------------------------
template <int KIND, int EPI>
__global__ __launch_bounds__(256) void ffn_gemm_f32(const GemmArgs p) {
  constexpr int T = 64, KS = 16;
  __shared__ float As[KS][T + 4];
  __shared__ float Bs[KS][T + 4];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int tile = blockIdx.x;
  const int tiles_per_g = p.tiles_m * p.tiles_n;
  const int g = tile / tiles_per_g;
  const int tr = tile - g * tiles_per_g;
  const int m0 = (tr / p.tiles_n) * T, n0 = (tr % p.tiles_n) * T;
  const float* __restrict__ A = reinterpret_cast<const float*>(p.A);
  const float* __restrict__ B = reinterpret_cast<const float*>(p.B);
  const int Kd = (KIND == KIND_TN) ? p.R : p.Kdim;
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;

  for (int k0 = 0; k0 < Kd; k0 += KS) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = tid + q * 256;  // 1024 elements per operand tile
      {
        // A tile element (i, k)
        int i, k;
        if (KIND == KIND_TN) { i = c & 63; k = c >> 6; } else { k = c & 15; i = c >> 4; }
        float v = 0.f;
        if (m0 + i < p.Mdim && k0 + k < Kd) {
          if (KIND == KIND_TN) v = A[phys_row(k0 + k, g, p.G, p.Cc) * p.lda + m0 + i];
          else v = A[phys_row(m0 + i, g, p.G, p.Cc) * p.lda + k0 + k];
        }
        As[k][i] = v;
      }
      {
        // B tile element (k, j)
        int j, k;
        if (KIND == KIND_NT) { k = c & 15; j = c >> 4; } else { j = c & 63; k = c >> 6; }
        float v = 0.f;
        if (n0 + j < p.Ndim && k0 + k < Kd) {
          if (KIND == KIND_NN) v = B[(int64_t)g * p.b_goff + p.b_off + (int64_t)(k0 + k) * p.ldb + n0 + j];
          else if (KIND == KIND_NT) v = B[(int64_t)g * p.b_goff + p.b_off + (int64_t)(n0 + j) * p.ldb + k0 + k];
          else v = B[phys_row(k0 + k, g, p.G, p.Cc) * p.ldb + n0 + j];
        }
        Bs[k][j] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
      const double ad[4] = {(double)a.x, (double)a.y, (double)a.z, (double)a.w};
      const double bd[4] = {(double)b.x, (double)b.y, (double)b.z, (double)b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fma(ad[i], bd[j], acc[i][j]);
    }
    __syncthreads();
  }
  float* __restrict__ C = reinterpret_cast<float*>(p.C);
  float* __restrict__ C2 = reinterpret_cast<float*>(p.C2);
  const float* __restrict__ Z = reinterpret_cast<const float*>(p.Zin);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= p.Mdim) continue;
    int64_t crow;
    if (KIND == KIND_TN) crow = (int64_t)g * p.c_goff + p.c_off + (int64_t)m * p.ldc;
    else crow = phys_row(m, g, p.G, p.Cc) * p.ldc;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= p.Ndim) continue;
      const float v = (float)acc[i][j];
      if (EPI == EPI_STORE) {
        C[crow + n] = v;
      } else if (EPI == EPI_GELU) {
        C[crow + n] = v;
        C2[crow + n] = gelu_f(v);
      } else {
        float ge, dg;
        gelu_and_grad(Z[crow + n], ge, dg);
        C[crow + n] = v * dg;
        C2[crow + n] = ge;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
int g_tile_pref = 0;  // 0 auto, 1 = 128x128, 2 = 256x256

template <int KIND, int EPI>
void launch_gemm(GemmArgs a, int dtype, hipStream_t st) {
  if (dtype == MOE_F32) {
    a.tiles_m = (a.Mdim + 63) / 64;
    a.tiles_n = (a.Ndim + 63) / 64;
    a.total_tiles = a.G * a.tiles_m * a.tiles_n;
    hipLaunchKernelGGL((ffn_gemm_f32<KIND, EPI>), dim3(a.total_tiles), dim3(256), 0, st, a);
    return;
  }
  a.kchunks = (a.Cc + KT - 1) / KT;
  const int64_t big_tiles = (int64_t)a.G * ((a.Mdim + 255) / 256) * ((a.Ndim + 255) / 256);
  bool big = big_tiles >= 512;
  if (g_tile_pref == 1) big = false;
  if (g_tile_pref == 2) big = true;
  const int T = big ? 256 : 128;
  a.tiles_m = (a.Mdim + T - 1) / T;
  a.tiles_n = (a.Ndim + T - 1) / T;
  a.total_tiles = a.G * a.tiles_m * a.tiles_n;
  const dim3 grid((unsigned)(((a.total_tiles + 7) / 8) * 8));
  if (big) hipLaunchKernelGGL((ffn_gemm_bf16<256, 256, 2, 2, KIND, EPI>), grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL((ffn_gemm_bf16<128, 128, 2, 2, KIND, EPI>), grid, dim3(256), 0, st, a);
}

int check_ffn_shape(int dtype, int n_src, int G, int64_t C, int M, int H, int esp_idx, int n_esp) {
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_EINVAL);
  MOE_REQUIRE(n_src >= 1 && G >= 1 && C >= 1 && M >= 1 && H >= 1, MOE_EINVAL);
  MOE_REQUIRE(n_esp >= 1 && esp_idx >= 0 && esp_idx < n_esp && H % n_esp == 0, MOE_EINVAL);
  const int Hl = H / n_esp;
  MOE_REQUIRE(M % 8 == 0 && Hl % 8 == 0, MOE_EUNSUPPORTED);
  MOE_REQUIRE((int64_t)n_src * C < (1ll << 31) && (int64_t)n_src * G * C < (1ll << 31), MOE_EUNSUPPORTED);
  return MOE_OK;
}

}  // namespace

extern "C" int moe_ffn_set_tile(int tile) {
  if (tile < 0 || tile > 2) return MOE_EINVAL;
  g_tile_pref = tile;
  return MOE_OK;
}

extern "C" size_t moe_ffn_workspace_bytes(int dtype, int n_src, int G, int64_t C, int M, int H, int n_esp,
                                          int backward) {
  if (check_ffn_shape(dtype, n_src, G, C, M, H, 0, n_esp) != MOE_OK) return 0;
  const size_t esz = dtype == MOE_BF16 ? 2 : 4;
  const size_t one = moe::align_up((size_t)n_src * G * C * (size_t)(H / n_esp) * esz, 256);
  return backward ? 2 * one : one;
}

extern "C" int moe_expert_ffn_fwd(const void* X, int dtype, const void* W1, const void* W2, int n_src, int G,
                                  int64_t C, int M, int H, int esp_idx, int n_esp, void* Z, void* Y, void* ws,
                                  size_t ws_bytes, void* stream) {
  if (int rc = check_ffn_shape(dtype, n_src, G, C, M, H, esp_idx, n_esp)) return rc;
  MOE_REQUIRE_PTR(X); MOE_REQUIRE_PTR(W1); MOE_REQUIRE_PTR(W2); MOE_REQUIRE_PTR(Z); MOE_REQUIRE_PTR(Y);
  const size_t need = moe_ffn_workspace_bytes(dtype, n_src, G, C, M, H, n_esp, 0);
  MOE_REQUIRE(ws != nullptr && ws_bytes >= need, MOE_EWORKSPACE);
  MOE_REQUIRE(moe::aligned16(ws), MOE_EALIGN);
  hipStream_t st = (hipStream_t)stream;
  const int Hl = H / n_esp;
  const int64_t h0 = (int64_t)esp_idx * Hl;
  void* Act = ws;

  GemmArgs a{};
  a.G = G; a.n_src = n_src; a.Cc = (int)C; a.R = (int)(n_src * C);
  // Z = X * W1[:, h0:h0+Hl]; Act = GeLU(Z)
  a.A = X; a.lda = M;
  a.B = W1; a.ldb = H; a.b_goff = (int64_t)M * H; a.b_off = h0;
  a.C = Z; a.C2 = Act; a.ldc = Hl;
  a.Mdim = a.R; a.Ndim = Hl; a.Kdim = M;
  launch_gemm<KIND_NN, EPI_GELU>(a, dtype, st);
  // Y = Act * W2[h0:h0+Hl, :]
  a.A = Act; a.lda = Hl;
  a.B = W2; a.ldb = M; a.b_goff = (int64_t)H * M; a.b_off = h0 * M;
  a.C = Y; a.C2 = nullptr; a.ldc = M;
  a.Mdim = a.R; a.Ndim = M; a.Kdim = Hl;
  launch_gemm<KIND_NN, EPI_STORE>(a, dtype, st);
  return moe::check_launch();
}

extern "C" int moe_expert_ffn_bwd(const void* dY, const void* X, const void* Z, const void* W1, const void* W2,
                                  int dtype, int n_src, int G, int64_t C, int M, int H, int esp_idx, int n_esp,
                                  void* dX, void* dW1, void* dW2, void* ws, size_t ws_bytes, void* stream) {
  if (int rc = check_ffn_shape(dtype, n_src, G, C, M, H, esp_idx, n_esp)) return rc;
  MOE_REQUIRE_PTR(dY); MOE_REQUIRE_PTR(X); MOE_REQUIRE_PTR(Z); MOE_REQUIRE_PTR(W1); MOE_REQUIRE_PTR(W2);
  MOE_REQUIRE_PTR(dX); MOE_REQUIRE_PTR(dW1); MOE_REQUIRE_PTR(dW2);
  const size_t need = moe_ffn_workspace_bytes(dtype, n_src, G, C, M, H, n_esp, 1);
  MOE_REQUIRE(ws != nullptr && ws_bytes >= need, MOE_EWORKSPACE);
  MOE_REQUIRE(moe::aligned16(ws), MOE_EALIGN);
  hipStream_t st = (hipStream_t)stream;
  const int Hl = H / n_esp;
  const int64_t h0 = (int64_t)esp_idx * Hl;
  void* Act = ws;
  void* dZ = (char*)ws + need / 2;

  GemmArgs a{};
  a.G = G; a.n_src = n_src; a.Cc = (int)C; a.R = (int)(n_src * C);
  // dA = dY * W2[h0:h0+Hl, :]^T ; dZ = dA * GeLU'(Z) ; Act = GeLU(Z)
  a.A = dY; a.lda = M;
  a.B = W2; a.ldb = M; a.b_goff = (int64_t)H * M; a.b_off = h0 * M;
  a.C = dZ; a.C2 = Act; a.Zin = Z; a.ldc = Hl;
  a.Mdim = a.R; a.Ndim = Hl; a.Kdim = M;
  launch_gemm<KIND_NT, EPI_DGELU>(a, dtype, st);
  // dW2[h0:h0+Hl, :] = Act^T * dY
  a.A = Act; a.lda = Hl;
  a.B = dY; a.ldb = M;
  a.C = dW2; a.C2 = nullptr; a.Zin = nullptr; a.ldc = M; a.c_goff = (int64_t)H * M; a.c_off = h0 * M;
  a.Mdim = Hl; a.Ndim = M; a.Kdim = a.R;
  launch_gemm<KIND_TN, EPI_STORE>(a, dtype, st);
  // dW1[:, h0:h0+Hl] = X^T * dZ
  a.A = X; a.lda = M;
  a.B = dZ; a.ldb = Hl;
  a.C = dW1; a.ldc = H; a.c_goff = (int64_t)M * H; a.c_off = h0;
  a.Mdim = M; a.Ndim = Hl; a.Kdim = a.R;
  launch_gemm<KIND_TN, EPI_STORE>(a, dtype, st);
  // dX = dZ * W1[:, h0:h0+Hl]^T
  a.A = dZ; a.lda = Hl;
  a.B = W1; a.ldb = H; a.b_goff = (int64_t)M * H; a.b_off = h0;
  a.C = dX; a.ldc = M; a.c_goff = 0; a.c_off = 0;
  a.Mdim = a.R; a.Ndim = M; a.Kdim = Hl;
  launch_gemm<KIND_NT, EPI_STORE>(a, dtype, st);
  return moe::check_launch();
}
