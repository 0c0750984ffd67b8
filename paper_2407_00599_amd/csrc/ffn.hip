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
// bf16 path: MFMA v_mfma_f32_32x32x16_bf16, fp32 accumulation, two kernels.
//   ffn_gemm_dma  (every problem with at least 64 tiles of 256 x 256): global memory goes straight to
//       LDS (buffer_load ... lds), a ring of five 32 KiB stages of k tile 32, 8 waves; operands whose
//       memory layout has k as the slow index stay in that layout in LDS and are read with the
//       transposing LDS load, so no transpose pass exists.  Described in front of gemm_dma_tile.
//   ffn_gemm_bf16 (small problems, 128 x 128 tiles): global -> registers -> LDS tiles [row][k] with
//       k contiguous (row pitch 64 + 8 bf16: conflict-free 16-byte fragment reads); operands with k as
//       the slow index are transposed in registers (8x8 blocks, v_perm) on their way to LDS; the loads
//       of k tile kt+1 are issued before the MFMAs of tile kt (LDS double buffer, one barrier per tile).
// Both issue the MFMA with the operands swapped (D^T = B^T A^T) so that a lane ends up with 4
// consecutive output columns.  Workgroup ids are remapped so that each XCD (ids are dealt round-robin
// to the 8 XCDs) works on one contiguous range of tiles and its L2 sees the same operand panels.
//
// fp32 path: a plain LDS-tiled kernel with fp64 accumulation, for the small fp32 configuration.
#include <type_traits>

#include "common.h"

namespace {

using namespace moe;

enum { KIND_NN = 1, KIND_NT = 2, KIND_TN = 3 };
enum { EPI_STORE = 0, EPI_GELU = 1, EPI_DGELU = 2 };

struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  void* C2;         // second output (the activation GeLU(Z)) for EPI_GELU
  const void* Zin;  // saved pre-activation for EPI_DGELU
  const int32_t* cnt;  // optional [n_src, G]: rows of chunk (s, g) at or beyond min(cnt, Cc) are zero padding
  // fused dispatch (NN GEMMs, n_src = 1): A is the token matrix and row r of expert g is the token
  // gather[g * Cc + r] / gather_k (the gate's inverse slot map; negative = empty slot, a zero row)
  const int32_t* gather;
  int gather_k;
  uint32_t gather_magic;  // ceil(2^32 / gather_k): v / gather_k = umulhi(v, magic) for v < 2^29 (gather_k <= 8)
  int64_t gather_rows;    // rows of the token matrix
  int G, n_src;
  int Cc;           // rows per chunk (capacity C)
  int R;            // n_src * Cc: virtual rows per expert
  int Mdim, Ndim, Kdim;
  int64_t lda, ldb, ldc;             // leading dimensions, elements
  int64_t b_goff, c_goff;            // per-expert stride of weight-type operands, elements
  int64_t b_off, c_off;              // constant offset of the ESP slice, elements
  int tiles_m, tiles_n, total_tiles;
  int kchunks;                       // TN: k tiles per chunk = ceil(Cc / 64)
  uint64_t a_bytes, b_bytes;         // bf16 path: byte sizes of the A and B tensors (buffer descriptors)
};

__device__ __forceinline__ int64_t phys_row(int r, int g, int G, int Cc) {
  const int s = r / Cc;
  return ((int64_t)s * G + g) * Cc + (r - s * Cc);
}

// Row of the A operand that virtual row r of expert g is read from: its place in the received layout,
// or, with a gather map, the token that the slot holds (-1: an empty slot, read as zeros).
__device__ __forceinline__ int64_t a_src_row(const GemmArgs& p, int r, int g) {
  if (p.gather == nullptr) return phys_row(r, g, p.G, p.Cc);
  const int iv = p.gather[(int64_t)g * p.Cc + r];
  if (iv < 0) return -1;
  const int64_t tok = iv / p.gather_k;
  return tok < p.gather_rows ? tok : -1;   // an index past the token matrix is treated as an empty slot
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

// Guarded 16-byte loads go through buffer descriptors: a lane that must not load passes an
// offset beyond num_records and receives zeros, without a branch, so the whole k loop body is
// one basic block whose loads, LDS traffic and MFMAs can be interleaved.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr uint32_t OOB = 0xFFFFFFF0u;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ void pin(uint4& v) {
  asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
}
template <bool STREAM = false>   // STREAM: non-temporal hint, for data read here for the last time
__device__ __forceinline__ uint4 ldb16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, STREAM ? 2 : 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// coefficients written by fit_gelu_poly.py (this directory)
__device__ constexpr float GELU_PHI[9] = {3.989023268e-01f, -6.634449214e-02f, 9.815968573e-03f, -1.108560129e-03f,
                                          9.341852274e-05f, -5.626405255e-06f, 2.255412426e-07f, -5.327701835e-09f,
                                          5.564777111e-11f};
__device__ constexpr float GELU_DG[10] = {7.977564335e-01f, -2.653926015e-01f, 5.909253657e-02f, -9.040454403e-03f,
                                          9.965471691e-04f, -7.936266047e-05f, 4.432653895e-06f, -1.634905260e-07f,
                                          3.552443228e-09f, -3.426744305e-11f};
// GeLU pieces for the bf16 epilogues, transcendental-free: on |z| <= 4.25 the odd parts of
//   Phi(z) - 1/2            (Phi = standard normal CDF, GeLU(z) = z Phi(z))   and
//   GeLU'(z) - 1/2 = Phi(z) + z phi(z) - 1/2
// are odd minimax polynomials in z (9 and 10 coefficients, fitted in fp64 and evaluated by Horner in
// fp32); outside that range z is clamped, where both functions are within 2e-4 of their limits.
// Evaluated in fp32: |GeLU error| < 5e-5 (relative 1e-5 for large z), |GeLU' error| < 1.7e-4, both far
// below the bf16 rounding of the stored result (2^-9 relative).
__device__ __forceinline__ float gelu_poly(float z) {
  const float zc = __builtin_amdgcn_fmed3f(z, -4.25f, 4.25f);
  const float u = zc * zc;
  float q = fmaf(GELU_PHI[8], u, GELU_PHI[7]);
#pragma unroll
  for (int i = 6; i >= 0; --i) q = fmaf(q, u, GELU_PHI[i]);
  const float cdf = __builtin_amdgcn_fmed3f(fmaf(zc, q, 0.5f), 0.0f, 1.0f);
  return z * cdf;
}
__device__ __forceinline__ float gelu_grad_poly(float z) {
  const float zc = __builtin_amdgcn_fmed3f(z, -4.25f, 4.25f);
  const float u = zc * zc;
  float q = fmaf(GELU_DG[9], u, GELU_DG[8]);
#pragma unroll
  for (int i = 7; i >= 0; --i) q = fmaf(q, u, GELU_DG[i]);
  return fmaf(zc, q, 0.5f);
}

// Epilogue shared by the bf16 kernels.  A lane holds, for each 32x32 block (i, j) of its wave
// tile, output row m = mbase + 32 i + lane%32 and columns n = nbase + 32 j + 8 (q/4) + 4 (lane/32)
// + q%4 for q = 0..15, i.e. four runs of 4 consecutive columns: 8-byte stores.
template <int MB, int NBK, int KIND, int EPI>
__device__ __forceinline__ void store_tile(const GemmArgs& p, f32x16_t (&acc)[MB][NBK], int g, int mbase, int nbase,
                                           int lane) {
  bf16_t* __restrict__ Cb = reinterpret_cast<bf16_t*>(p.C);
  bf16_t* __restrict__ C2b = reinterpret_cast<bf16_t*>(p.C2);
  const bf16_t* __restrict__ Zb = reinterpret_cast<const bf16_t*>(p.Zin);
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    const int m = mbase + i * 32 + (lane & 31);
    if (m >= p.Mdim) continue;
    int64_t crow;
    if (KIND == KIND_TN) crow = (int64_t)g * p.c_goff + p.c_off + (int64_t)m * p.ldc;
    else crow = phys_row(m, g, p.G, p.Cc) * p.ldc;
#pragma unroll
    for (int j = 0; j < NBK; ++j) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int n = nbase + j * 32 + q4 * 8 + (lane >> 5) * 4;
        if (n >= p.Ndim) continue;
        float v[4] = {acc[i][j][q4 * 4 + 0], acc[i][j][q4 * 4 + 1], acc[i][j][q4 * 4 + 2], acc[i][j][q4 * 4 + 3]};
        if (EPI == EPI_STORE) {
          *reinterpret_cast<uint2*>(Cb + crow + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        } else if (EPI == EPI_GELU) {
          *reinterpret_cast<uint2*>(Cb + crow + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          float a[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) a[e] = gelu_poly(v[e]);
          *reinterpret_cast<uint2*>(C2b + crow + n) = make_uint2(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]));
        } else {
          const uint2 zq = *reinterpret_cast<const uint2*>(Zb + crow + n);
          const float z[4] = {__uint_as_float(zq.x << 16), __uint_as_float(zq.x & 0xFFFF0000u),
                              __uint_as_float(zq.y << 16), __uint_as_float(zq.y & 0xFFFF0000u)};
          float d[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) d[e] = v[e] * gelu_grad_poly(z[e]);
          *reinterpret_cast<uint2*>(Cb + crow + n) = make_uint2(pack_bf16x2(d[0], d[1]), pack_bf16x2(d[2], d[3]));
        }
      }
    }
  }
}

// Workgroup -> output tile.  Workgroup ids are dealt round-robin to the 8 XCDs, so id % 8 names
// the XCD; each XCD is given one contiguous range of a linear tile order in which 32 consecutive
// tiles (what its 32 CUs run at the same time) form an 8 (rows) x 4 (columns) patch of one expert:
// per k step they share 8 + 4 operand slices in that XCD's L2 instead of 1 + 32.
// (vb = index of the workgroup within its problem; problems of a merged launch start at multiples of 8,
// so vb % 8 is still the XCD)
__device__ __forceinline__ bool map_tile(const GemmArgs& p, int vb, int& g, int& tm, int& tn) {
  constexpr int SW = 4;
  const int per_xcd = (p.total_tiles + 7) / 8;
  const int tile = (vb & 7) * per_xcd + (vb >> 3);
  if (tile >= p.total_tiles) return false;
  const int tiles_per_g = p.tiles_m * p.tiles_n;
  g = tile / tiles_per_g;
  const int t = tile - g * tiles_per_g;
  const int full = p.tiles_n / SW;
  const int strip = p.tiles_m * SW;
  if (t < full * strip) {
    const int sn = t / strip, r = t - sn * strip;
    tm = r / SW;
    tn = sn * SW + (r - tm * SW);
  } else {
    const int w = p.tiles_n - full * SW;
    const int r = t - full * strip;
    tm = r / w;
    tn = full * SW + (r - tm * w);
  }
  return true;
}

// Instruction-order hints for the scheduler (sched_group_barrier): "N instructions of this
// class next".  Recipe interleaves NM MFMAs with NA instructions of class MA and NB of class MB.
enum { SG_MFMA = 0x008, SG_VMEM_READ = 0x020, SG_DS_READ = 0x100, SG_DS_WRITE = 0x200 };
template <int MASK, int N>
__device__ __forceinline__ void sched_group() {
  if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}
template <int I, int NM, int NA, int MA, int NB, int MB_>
struct Recipe {
  static __device__ __forceinline__ void run() {
    if constexpr (I < NM) {
      sched_group<MA, (I + 1) * NA / NM - I * NA / NM>();
      sched_group<MB_, (I + 1) * NB / NM - I * NB / NM>();
      sched_group<SG_MFMA, 1>();
      Recipe<I + 1, NM, NA, MA, NB, MB_>::run();
    }
  }
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

  int g, tm, tn;
  if (!map_tile(p, (int)blockIdx.x, g, tm, tn)) return;
  const int m0 = tm * TM, n0 = tn * TN;

  const int64_t b_base = (int64_t)g * p.b_goff + p.b_off;   // weight-type B: start of expert g's slice
  // descriptors: activation tensors whole (host guarantees < 4 GiB); weights from expert g's slice on
  const __amdgpu_buffer_rsrc_t rA = make_rsrc(p.A, (uint32_t)p.a_bytes);
  const uint64_t b_rem = p.b_bytes - (uint64_t)b_base * 2;
  const __amdgpu_buffer_rsrc_t rB =
      (KIND == KIND_TN) ? make_rsrc(p.B, (uint32_t)p.b_bytes)
                        : make_rsrc(reinterpret_cast<const bf16_t*>(p.B) + b_base,
                                    b_rem > OOB ? OOB : (uint32_t)b_rem);

  // ---- per-thread staging coordinates (fixed over the k loop), byte offsets ----
  // direct:      chunk i -> row = tid/8 + i*(NT/8), k chunk = tid%8
  // transposed:  full 8x8 blocks: bi = tid + b*NT, kb = bi%8, r8 = bi/8;  half blocks: kb4 = tid%16, r8 = tid/16
  uint32_t a_off[A_TR ? 1 : SA::NCH];
  if (!A_TR) {
#pragma unroll
    for (int i = 0; i < SA::NCH; ++i) {
      const int r = m0 + (tid >> 3) + i * (NT / 8);
      const int64_t row = (r < p.Mdim) ? a_src_row(p, r, g) : -1;
      a_off[i] = (row >= 0) ? (uint32_t)((row * p.lda + (tid & 7) * 8) * 2) : OOB;
    }
  }
  uint32_t b_off[B_TR ? 1 : SB::NCH];
  if (!B_TR) {
#pragma unroll
    for (int i = 0; i < SB::NCH; ++i) {
      const int n = n0 + (tid >> 3) + i * (NT / 8);
      b_off[i] = (n < p.Ndim) ? (uint32_t)(((int64_t)n * p.ldb + (tid & 7) * 8) * 2) : OOB;
    }
  }
  const int nk = (KIND == KIND_TN) ? p.n_src * p.kchunks : (p.Kdim + KT - 1) / KT;
  const uint32_t lda2 = (uint32_t)(p.lda * 2), ldb2 = (uint32_t)(p.ldb * 2);

  SA sa;
  SB sb;

  // global -> registers for k tile kt; kt >= nk loads nothing (all lanes out of range)
  auto load_tiles = [&](int kt) {
    const bool live = kt < nk;
    // ---------------- A ----------------
    if (!A_TR) {
      const int k0 = kt * KT;
      const bool kok = live && k0 + (tid & 7) * 8 < p.Kdim;
#pragma unroll
      for (int i = 0; i < SA::NCH; ++i)
        sa.reg[i] = ldb16(rA, (kok && a_off[i] != OOB) ? a_off[i] + (uint32_t)k0 * 2u : OOB);
    } else {
      const int s = kt / p.kchunks;
      const int c0 = (kt - s * p.kchunks) * KT;
      const int64_t chunk_row = ((int64_t)s * p.G + g) * p.Cc + c0;
      const int klim = live ? p.Cc - c0 : 0;
      if (!SA::HALF) {
#pragma unroll
        for (int b = 0; b < SA::NB; ++b) {
          const int bi = tid + b * NT;
          const int kb = bi & 7, r8 = bi >> 3;
          const int col = m0 + r8 * 8;
          const uint32_t off0 = (uint32_t)(((chunk_row + kb * 8) * p.lda + col) * 2);
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            uint32_t o = off0 + i * lda2;
            bool ok = kb * 8 + i < klim && col < p.Mdim;
            if (p.gather != nullptr && ok) {   // fused dispatch: the row is a token looked up through the slot map
              const int64_t row = a_src_row(p, c0 + kb * 8 + i, g);
              ok = row >= 0;
              o = (uint32_t)((row * p.lda + col) * 2);
            }
            sa.reg[b * 8 + i] = ldb16(rA, ok ? o : OOB);
          }
        }
      } else {
        const int kb4 = tid & 15, r8 = tid >> 4;
        const int col = m0 + r8 * 8;
        const uint32_t off0 = (uint32_t)(((chunk_row + kb4 * 4) * p.lda + col) * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          uint32_t o = off0 + i * lda2;
          bool ok = kb4 * 4 + i < klim && col < p.Mdim;
          if (p.gather != nullptr && ok) {
            const int64_t row = a_src_row(p, c0 + kb4 * 4 + i, g);
            ok = row >= 0;
            o = (uint32_t)((row * p.lda + col) * 2);
          }
          sa.reg[i] = ldb16(rA, ok ? o : OOB);
        }
      }
    }
    // ---------------- B ----------------
    if (!B_TR) {  // NT: weight rows n, k contiguous
      const int k0 = kt * KT;
      const bool kok = live && k0 + (tid & 7) * 8 < p.Kdim;
#pragma unroll
      for (int i = 0; i < SB::NCH; ++i)
        sb.reg[i] = ldb16(rB, (kok && b_off[i] != OOB) ? b_off[i] + (uint32_t)k0 * 2u : OOB);
    } else {
      uint32_t krow0;  // byte offset of k row 0 of this tile (relative to the descriptor base)
      int klim;        // number of valid k rows in this tile
      if (KIND == KIND_NN) {
        krow0 = (uint32_t)((int64_t)kt * KT * p.ldb * 2);
        klim = live ? p.Kdim - kt * KT : 0;
      } else {
        const int s = kt / p.kchunks;
        const int c0 = (kt - s * p.kchunks) * KT;
        krow0 = (uint32_t)((((int64_t)s * p.G + g) * p.Cc + c0) * p.ldb * 2);
        klim = live ? p.Cc - c0 : 0;
      }
      if (!SB::HALF) {
#pragma unroll
        for (int b = 0; b < SB::NB; ++b) {
          const int bi = tid + b * NT;
          const int kb = bi & 7, r8 = bi >> 3;
          const int col = n0 + r8 * 8;
          const uint32_t off0 = krow0 + (uint32_t)(kb * 8) * ldb2 + (uint32_t)col * 2u;
#pragma unroll
          for (int i = 0; i < 8; ++i)
            sb.reg[b * 8 + i] = ldb16(rB, (kb * 8 + i < klim && col < p.Ndim) ? off0 + i * ldb2 : OOB);
        }
      } else {
        const int kb4 = tid & 15, r8 = tid >> 4;
        const int col = n0 + r8 * 8;
        const uint32_t off0 = krow0 + (uint32_t)(kb4 * 4) * ldb2 + (uint32_t)col * 2u;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          sb.reg[i] = ldb16(rB, (kb4 * 4 + i < klim && col < p.Ndim) ? off0 + i * ldb2 : OOB);
      }
    }
  };

  auto store_A = [&](int buf) {
    bf16_t* As = smem + buf * (TM + TN) * PITCH;
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
  };
  auto store_B = [&](int buf) {
    bf16_t* Bs = smem + buf * (TM + TN) * PITCH + TM * PITCH;
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

  // fragment addresses of this lane inside a stage
  const int a_frag = (wm * TMW + (lane & 31)) * PITCH + (lane >> 5) * 8;
  const int b_frag = TM * PITCH + (wn * TNW + (lane & 31)) * PITCH + (lane >> 5) * 8;
  bf16x8_t fa[2][MB], fb[2][NBK];
  auto load_frags = [&](int buf, int kk, int set) {
    const bf16_t* st = smem + buf * (TM + TN) * PITCH + kk * 16;
#pragma unroll
    for (int i = 0; i < MB; ++i) fa[set][i] = *reinterpret_cast<const bf16x8_t*>(st + a_frag + i * 32 * PITCH);
#pragma unroll
    for (int j = 0; j < NBK; ++j) fb[set][j] = *reinterpret_cast<const bf16x8_t*>(st + b_frag + j * 32 * PITCH);
  };

  constexpr int NWA = A_TR ? 8 * (SA::HALF ? 1 : SA::NB) : SA::NCH;   // LDS writes per tile, A / B
  constexpr int NWB = B_TR ? 8 * (SB::HALF ? 1 : SB::NB) : SB::NCH;
  load_tiles(0);
  store_A(0);
  store_B(0);
  __syncthreads();
  load_frags(0, 0, 0);

  // One k tile per iteration; the body is branch-free.  sched_barrier(0) fences keep the order
  // written here: global loads of the next tile first (a whole tile of MFMAs hides their
  // latency), fragment reads of step kk+1 issued before the MFMAs of step kk, LDS writes of the
  // next tile riding on the last two MFMA groups.
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
      const int cur = kk & 1;
      if (kk + 1 < KT / 16) load_frags(buf, kk + 1, cur ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      if (kk == 0) load_tiles(kt + 1);
      // the empty asm pins the staged registers here, so the transposes that consume them are
      // not hoisted up to the loads (where they would wait for memory)
      if (kk == KT / 16 - 2) {
#pragma unroll
        for (int i = 0; i < SA::NCH; ++i) pin(sa.reg[i]);
        store_A(buf ^ 1);
      }
      if (kk == KT / 16 - 1) {
#pragma unroll
        for (int i = 0; i < SB::NCH; ++i) pin(sb.reg[i]);
        store_B(buf ^ 1);
      }
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NBK; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
      // inside the fenced group: one memory instruction per MFMA, so that issuing the loads /
      // LDS writes never holds up the matrix pipe
      constexpr int NM = MB * NBK;
      if (kk == 0) Recipe<0, NM, SA::NCH + SB::NCH, SG_VMEM_READ, 0, SG_DS_READ>::run();
      if (kk == KT / 16 - 2) Recipe<0, NM, NWA, SG_DS_WRITE, 0, SG_DS_READ>::run();
      if (kk == KT / 16 - 1) Recipe<0, NM, NWB, SG_DS_WRITE, 0, SG_DS_READ>::run();
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    load_frags(buf ^ 1, 0, 0);
  }

  store_tile<MB, NBK, KIND, EPI>(p, acc, g, m0 + wm * TMW, n0 + wn * TNW, lane);
}

// Epilogue of the DMA kernel, staged through LDS so that global memory sees 16-byte accesses in
// which consecutive lanes cover a contiguous run of a row (the MFMA result layout alone gives
// 8-byte pieces strided across 32 rows).  Each wave owns a private slice of the (now idle) stage
// memory: per 32-row block it writes bf16 results in [32][CW] row-major form (CW = columns of the
// wave tile, row pitch 2 CW + 16 bytes), reads them back row-wise and stores them; the GeLU
// epilogue stages its second output, and the GeLU' epilogue the saved pre-activation it reads, the
// same way.  Global memory is addressed through buffer descriptors with 32-bit byte offsets, so
// the code is branch-free: a row or column outside the problem gets an out-of-range offset, which
// the hardware drops (stores) or answers with zeros (loads).
// STREAM = the non-temporal hint, for tensors that are not read again soon (the saved pre-activation,
// the weight gradients): they then do not push the weights and the live activations out of the
// last-level cache, which the next GEMMs read their operands from.
template <bool STREAM = false>
__device__ __forceinline__ void stb16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, const uint4& v) {
  const u32x4_t q = {v.x, v.y, v.z, v.w};
  __builtin_amdgcn_raw_buffer_store_b128(q, r, (int)byte_off, 0, STREAM ? 2 : 0);
}
template <int KIND, int EPI, int MB, int NBK>
__device__ __forceinline__ void store_tile_lds(const GemmArgs& p, f32x16_t (&acc)[MB][NBK], char* wave_lds, int g,
                                               int mbase, int nbase, int lane, bool zero_fill = false) {
  constexpr int CW = 32 * NBK;            // columns of the wave tile
  constexpr int PITCH_B = 2 * CW + 16;    // staged row pitch, bytes
  constexpr int BUF = 32 * PITCH_B;
  constexpr int LPR = CW / 8;             // lanes per row in the row-wise phase (16 bytes each)
  constexpr int RPI = 64 / LPR;           // rows per instruction
  constexpr int NT_ = 32 / RPI;           // instructions per 32-row block
  char* buf0 = wave_lds;          // first output (or staged Z on the way in)
  char* buf1 = wave_lds + BUF;    // second output
  const int rl = lane / LPR;      // row-wise phase: row RPI t + rl, 16-byte chunk lane % LPR
  const int cc = lane % LPR;
  const int ncol = nbase + cc * 8;
  const bool col_ok = ncol < p.Ndim;

  // descriptors: the activation tensors as a whole, or (weight gradients) this expert's matrix from
  // the first element of the shard on
  __amdgpu_buffer_rsrc_t rC, rC2, rZ;
  if (KIND == KIND_TN) {
    const uint32_t bytes = (uint32_t)(((int64_t)(p.Mdim - 1) * p.ldc + p.Ndim) * 2);
    rC = make_rsrc(reinterpret_cast<bf16_t*>(p.C) + ((int64_t)g * p.c_goff + p.c_off), bytes);
    rC2 = rC; rZ = rC;
  } else {
    const uint32_t bytes = (uint32_t)((uint64_t)p.n_src * p.G * p.Cc * (uint64_t)p.ldc * 2);
    rC = make_rsrc(p.C, bytes);
    rC2 = make_rsrc(EPI == EPI_GELU ? p.C2 : p.C, bytes);
    rZ = make_rsrc(EPI == EPI_DGELU ? p.Zin : p.C, bytes);
  }
  // byte offset of (row, ncol) for the rows this lane touches in the row-wise phase, or OOB.  One
  // multiplication per lane; the rows of a wave tile are then a constant number of leading dimensions apart.
  uint32_t off[MB][NT_];
  const uint32_t ldc2 = (uint32_t)p.ldc * 2u;
  if (KIND == KIND_TN) {
    const uint32_t base = ((uint32_t)(mbase + rl) * (uint32_t)p.ldc + (uint32_t)ncol) * 2u;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int t = 0; t < NT_; ++t) {
        const int d = i * 32 + RPI * t;
        off[i][t] = (mbase + d + rl < p.Mdim && col_ok) ? base + (uint32_t)d * ldc2 : OOB;
      }
  } else {
    // virtual row r of expert g is physical row ((r / C) G + g) C + r % C; one division for the
    // wave tile (a wave tile crosses at most one chunk boundary if C is not smaller than its
    // height: rows past it lie (G - 1) C physical rows further on)
    const int q0 = mbase / p.Cc, r0 = mbase - q0 * p.Cc;
    if (p.Cc >= 32 * MB) {
      const uint32_t row0 = (uint32_t)((q0 * p.G + g) * p.Cc + r0 + rl);
      const uint32_t base = (row0 * (uint32_t)p.ldc + (uint32_t)ncol) * 2u;
      const uint32_t wrap_add = (uint32_t)(p.G - 1) * (uint32_t)p.Cc * ldc2;
      const int to_wrap = p.Cc - r0 - rl;     // rows at or beyond this distance are in the next chunk
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int t = 0; t < NT_; ++t) {
          const int d = i * 32 + RPI * t;
          const uint32_t o = base + (uint32_t)d * ldc2 + (d >= to_wrap ? wrap_add : 0u);
          off[i][t] = (mbase + d + rl < p.Mdim && col_ok) ? o : OOB;
        }
    } else {
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int t = 0; t < NT_; ++t) {
          const int m = mbase + i * 32 + RPI * t + rl;
          const uint32_t row = (uint32_t)phys_row(m < p.Mdim ? m : 0, g, p.G, p.Cc);
          off[i][t] = (m < p.Mdim && col_ok) ? (row * (uint32_t)p.ldc + (uint32_t)ncol) * 2u : OOB;
        }
    }
  }
  if (zero_fill) {   // a tile of padding rows: every result is zero
    const uint4 z = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int t = 0; t < NT_; ++t) {
        stb16(rC, off[i][t], z);
        if (EPI == EPI_GELU) stb16(rC2, off[i][t], z);
      }
    return;
  }
  // accumulator phase: row lane % 32, for block j and q4: 4 columns at 32 j + 8 q4 + 4 (lane / 32)
  const int acc_off = (lane & 31) * PITCH_B + (lane >> 5) * 8;
#pragma unroll
  for (int i = 0; i < MB; ++i) {
    if (EPI == EPI_DGELU) {  // bring in the saved pre-activation, row-wise
#pragma unroll
      for (int t = 0; t < NT_; ++t)
        *reinterpret_cast<uint4*>(buf0 + (RPI * t + rl) * PITCH_B + cc * 16) = ldb16<true>(rZ, off[i][t]);
    }
#pragma unroll
    for (int j = 0; j < NBK; ++j) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float v[4] = {acc[i][j][q4 * 4 + 0], acc[i][j][q4 * 4 + 1], acc[i][j][q4 * 4 + 2], acc[i][j][q4 * 4 + 3]};
        char* a0 = buf0 + acc_off + j * 64 + q4 * 16;
        char* a1 = buf1 + acc_off + j * 64 + q4 * 16;
        if (EPI == EPI_STORE) {
          *reinterpret_cast<uint2*>(a0) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        } else if (EPI == EPI_GELU) {
          float a[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) a[e] = gelu_poly(v[e]);
          *reinterpret_cast<uint2*>(a0) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          *reinterpret_cast<uint2*>(a1) = make_uint2(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]));
        } else {
          const uint2 zq = *reinterpret_cast<const uint2*>(a0);
          const float z[4] = {__uint_as_float(zq.x << 16), __uint_as_float(zq.x & 0xFFFF0000u),
                              __uint_as_float(zq.y << 16), __uint_as_float(zq.y & 0xFFFF0000u)};
          float d[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) d[e] = v[e] * gelu_grad_poly(z[e]);
          *reinterpret_cast<uint2*>(a0) = make_uint2(pack_bf16x2(d[0], d[1]), pack_bf16x2(d[2], d[3]));
        }
      }
    }
    // row-wise read-back and store (LDS operations of one wave complete in program order)
#pragma unroll
    for (int t = 0; t < NT_; ++t) {
      stb16<(EPI == EPI_GELU || KIND == KIND_TN)>(rC, off[i][t],
                                                   *reinterpret_cast<const uint4*>(buf0 + (RPI * t + rl) * PITCH_B + cc * 16));
      if (EPI == EPI_GELU)
        stb16(rC2, off[i][t], *reinterpret_cast<const uint4*>(buf1 + (RPI * t + rl) * PITCH_B + cc * 16));
    }
  }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel with an LDS-DMA pipeline (the fast path for large GEMMs).
//
// 256x256 (or 192x256) output tile, 8 waves (2 along the rows x 4 along the columns, two per SIMD: 128x64 or
// 96x64 per wave), k tile 32, a ring of DSTAGES = 5 LDS stages of 32 KiB (all of a compute unit's LDS).
// Global memory goes straight to LDS (buffer_load ... lds, 16 bytes per lane, no VGPR staging, no
// ds_write): a wave instruction fills 1 KiB of consecutive 16-byte slots in lane order, so the
// tile is stored unpadded and bank conflicts are avoided by permuting WHICH 16-byte chunk of a
// row each lane fetches (an XOR swizzle that the fragment reads undo).  Lanes whose row / column
// / k index is out of range pass an out-of-range buffer offset; the hardware then writes zeros.
//   operand with k contiguous in memory : stage holds [row][32 k] (64 B rows, 4 chunks), chunk c
//       of row r sits in slot c ^ ((r >> 2) & 3); fragments are read with ds_read_b128.
//   operand with k as the slow index    : stage holds [32 k][256 cols] (512 B rows, 32 chunks),
//       chunk c of k-row k sits in slot c ^ (4 (k & 3)); fragments are read with the transposing
//       LDS load ds_read_b64_tr_b16: a 16-lane group reads a 4(k) x 16(col) patch (lane s: k-row
//       s/4, 8-byte piece s%4) and lane i receives the 4 k-values of column i.
// Pipeline: while tile t is multiplied, the B-operand requests of tile t+3 go out during its first
// 16-wide MFMA step and the A-operand requests of tile t+4 during its second.  Once per k tile, between
// the two steps, each wave waits until its own requests for tile t+1 have landed (s_waitcnt vmcnt),
// all waves meet at a barrier, and the stage freed by tile t-1 (the one tile t+4 goes to) may be
// refilled.  Because the barrier sits in the middle, the first fragments of tile t+1 are fetched under
// the second MFMA step and no LDS latency is exposed at the tile boundary.
// ------------------------------------------------------------------------------------------
#define LDS_AS __attribute__((address_space(3)))
typedef short s16x4_t __attribute__((ext_vector_type(4)));

constexpr int DT = 256;                    // tile edge
constexpr int DK = 32;                     // k tile
constexpr int DSTAGES = 5;                 // 160 KiB: all of a compute unit's LDS
// s_waitcnt immediate that waits until at most n vector-memory operations are outstanding (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }
constexpr int DREGION = DT * DK * 2;       // bytes per operand per stage (16 KiB)
constexpr int DSTAGE = 2 * DREGION;

__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t r, bf16_t* lds_wave_base, uint32_t byte_off) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (LDS_AS void*)lds_wave_base, 16, (int)byte_off, 0, 0, 0);
}
// Fragment reads are issued as volatile asm: the compiler then neither reorders them nor guards
// them with conservative waits against the LDS-DMA requests in flight.  The kernel waits for them
// itself (s_waitcnt lgkmcnt(0)) and passes the registers through ready() before the MFMAs use them.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
union Frag {
  bf16x8_t v;
  u32x4_t q;
  u32x2_t h[2];
};
template <int OFF>
__device__ __forceinline__ void lds_read_kc(Frag& f, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.q) : "v"(addr), "n"(OFF));
}
template <int OFF>
__device__ __forceinline__ void lds_read_nc(Frag& f, uint32_t addr_lo, uint32_t addr_hi) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.h[0]) : "v"(addr_lo), "n"(OFF));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.h[1]) : "v"(addr_hi), "n"(OFF));
}
__device__ __forceinline__ void ready(Frag& f) { asm volatile("" : "+v"(f.q)); }

// WN = waves along n: 4 (8 waves, 128x64 per wave, two per SIMD) is what is launched; the template also
// allows 2 (4 waves, 128x128 per wave).
// TMR = rows of the output tile: 256, or 192 (three 32-row blocks per wave; only for operands A
// with k contiguous) for problems whose 256-row tiling would leave many compute units idle.
template <int KIND, int EPI, int WN, int TMR, bool GATHER = false>
__device__ __forceinline__ void gemm_dma_tile(const GemmArgs& p, char* smem, int vb) {
  constexpr bool A_NC = (KIND == KIND_TN);                     // A has k as the slow index
  constexpr bool B_NC = (KIND == KIND_NN || KIND == KIND_TN);  // B has k as the slow index
  static_assert(TMR == 256 || (TMR == 192 && !A_NC && WN == 4), "unsupported tile height");
  // GATHER: the k-slow A operand of a weight-gradient GEMM (X^T dZ) is the token matrix read through the
  // inverse slot map (row r of the chunk is token gather[g C + r] / gather_k); n_src = 1.
  static_assert(!GATHER || (KIND == KIND_TN && WN == 4), "row gather in the reduction: the 8-wave weight-gradient kernel only");
  constexpr int MB = TMR / 64, NBK = 8 / WN;     // 32x32 blocks per wave tile
  constexpr int RPW = 8 / WN;             // requests per wave per operand per k tile (16 in all)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS bases in SGPRs
  const int wm = wave / WN, wn = wave % WN;

  int g, tm, tn;
  if (!map_tile(p, vb, g, tm, tn)) return;
  const int m0 = tm * TMR, n0 = tn * DT;

  const int64_t b_base = (int64_t)g * p.b_goff + p.b_off;
  const __amdgpu_buffer_rsrc_t rA = make_rsrc(p.A, (uint32_t)p.a_bytes);
  const uint64_t b_rem = p.b_bytes - (uint64_t)b_base * 2;
  const __amdgpu_buffer_rsrc_t rB =
      (KIND == KIND_TN) ? make_rsrc(p.B, (uint32_t)p.b_bytes)
                        : make_rsrc(reinterpret_cast<const bf16_t*>(p.B) + b_base, b_rem > OOB ? OOB : (uint32_t)b_rem);

  // Rows at or beyond a chunk's count are padding (zero inputs, zero results).  A row tile made of
  // nothing else stores zeros and leaves; a reduction over the rows (the weight gradients) stops at
  // the count when there is a single chunk.
  int kvalid = p.Cc;   // TN: rows of a chunk that are multiplied
  if (KIND == KIND_TN && p.cnt != nullptr && p.n_src == 1) kvalid = min(max(p.cnt[g], 0), p.Cc);
  const int kpc = max((kvalid + DK - 1) / DK, 1);  // TN: k tiles per chunk
  const int nk = (KIND == KIND_TN) ? (kvalid > 0 ? p.n_src * kpc : 0) : (p.Kdim + DK - 1) / DK;

  // ---- per-lane request coordinates: each wave issues RPW requests per operand per k tile ----
  // k-contiguous operand, request q = RPW wave + j: rows 16 q + lane/4, slot lane%4 holds logical chunk kc_c
  const int kc_c = (lane & 3) ^ ((lane >> 4) & 3);
  // k-slow operand, request q: k-rows 2 q + lane/32, slot lane%32 holds logical chunk nc_c[j]
  uint32_t a_req[RPW], b_req[RPW];   // byte offset of the lane's 16 bytes at k tile 0, or OOB
  int a_k[RPW], b_k[RPW];            // k index (within the k tile) this request covers (k-slow), or first k (k-contig)
#pragma unroll
  for (int j = 0; j < RPW; ++j) {
    const int q = wave * RPW + j;
    if (!A_NC) {
      const int rt = q * 16 + (lane >> 2);   // rows past a 192-row tile are never fetched
      const int r = m0 + rt;
      a_k[j] = kc_c * 8;
      const int64_t row = (rt < TMR && r < p.Mdim) ? a_src_row(p, r, g) : -1;
      a_req[j] = (row >= 0) ? (uint32_t)((row * p.lda + kc_c * 8) * 2) : OOB;
    } else {
      const int k = 2 * q + (lane >> 5);
      const int col = m0 + (((lane & 31) ^ (4 * (k & 3))) * 8);
      a_k[j] = k;
      a_req[j] = (col < p.Mdim) ? (uint32_t)(((int64_t)(GATHER ? 0 : k) * p.lda + col) * 2) : OOB;
    }
    if (!B_NC) {
      const int n = n0 + q * 16 + (lane >> 2);
      b_k[j] = kc_c * 8;
      b_req[j] = (n < p.Ndim) ? (uint32_t)(((int64_t)n * p.ldb + kc_c * 8) * 2) : OOB;
    } else {
      const int k = 2 * q + (lane >> 5);
      const int col = n0 + (((lane & 31) ^ (4 * (k & 3))) * 8);
      b_k[j] = k;
      b_req[j] = (col < p.Ndim) ? (uint32_t)(((int64_t)k * p.ldb + col) * 2) : OOB;
    }
  }

  // GATHER: the four k-rows a wave requests per k tile (4 wave .. 4 wave + 3: requests j = 0, 1, lane halves)
  // are the same for all its lanes, so their slot-map entries are read with scalar loads (issued as asm so
  // that they stay scalar: nothing is added to the vector-memory queue whose length the waits below count).
  // They are issued at the start of a k tile, have arrived at its second fragment wait (lgkmcnt(0)), and are
  // turned into per-lane row offsets after the barrier, just before the A request that uses them.
  uint32_t g_now[RPW];   // byte offset of the token row behind this lane's k-row of the next A request, or OOB
  auto gather_fetch = [&](int kt, int (&dst)[4]) {
    const int64_t last = (int64_t)p.G * p.Cc - 1;
    const int64_t i0 = (int64_t)g * p.Cc + kt * DK + 4 * wave;   // rows past the count are never used
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = i0 + u < last ? i0 + u : last;
      const uint32_t off = (uint32_t)__builtin_amdgcn_readfirstlane((int)(i * 4));
      asm volatile("s_load_dword %0, %1, %2" : "=s"(dst[u]) : "s"(p.gather), "s"(off));
    }
  };
  auto gather_rows = [&](int (&src)[4]) {   // after an lgkmcnt(0) wait that follows the fetch
#pragma unroll
    for (int u = 0; u < 4; ++u) asm volatile("" : "+s"(src[u]));
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
      const int iv = (lane >> 5) ? src[2 * j + 1] : src[2 * j];
      const uint32_t tok = p.gather_k == 1 ? (uint32_t)iv : __umulhi((uint32_t)iv, p.gather_magic);
      g_now[j] = (iv >= 0 && (int64_t)tok < p.gather_rows) ? tok * (uint32_t)(p.lda * 2) : OOB;
    }
  };
  // Requests of k tile kt into its stage, one instruction (1 KiB) at a time: which = 0 (A) / 1 (B),
  // j = 0..RPW-1.  Tiles past the end still issue (all lanes out of range, zeros are written) so that
  // the number of outstanding requests per wave is the same in every iteration.
  auto request1 = [&](int kt, int stage, int which, int j) {
    char* st = smem + stage * DSTAGE;
    const bool live = kt < nk;
    uint32_t add;   // byte offset of the k tile
    int lim;        // valid k count in this tile
    if (KIND == KIND_TN) {
      const int s = kt / kpc;
      const int c0 = (kt - s * kpc) * DK;
      const int64_t row0 = ((int64_t)s * p.G + g) * p.Cc + c0;
      add = (uint32_t)(row0 * (which ? p.ldb : p.lda) * 2);
      lim = live ? kvalid - c0 : 0;
    } else {
      add = (which && B_NC) ? (uint32_t)((int64_t)kt * DK * p.ldb * 2) : (uint32_t)kt * (DK * 2);
      lim = live ? p.Kdim - kt * DK : 0;
    }
    const int q = wave * RPW + j;
    if (which == 0) {
      if (GATHER)
        dma16(rA, reinterpret_cast<bf16_t*>(st + q * 1024),
              (a_req[j] != OOB && g_now[j] != OOB && a_k[j] < lim) ? a_req[j] + g_now[j] : OOB);
      else
        dma16(rA, reinterpret_cast<bf16_t*>(st + q * 1024), (a_req[j] != OOB && a_k[j] < lim) ? a_req[j] + add : OOB);
    }
    else
      dma16(rB, reinterpret_cast<bf16_t*>(st + DREGION + q * 1024),
            (b_req[j] != OOB && b_k[j] < lim) ? b_req[j] + add : OOB);
  };
  auto request_half = [&](int kt, int which) {   // prologue only: kt < DSTAGES
#pragma unroll
    for (int j = 0; j < RPW; ++j) request1(kt, kt, which, j);
  };

  // ---- per-lane fragment addresses inside a stage (bytes), for k step kk = 0; kk = 1 adds a constant ----
  // k-contiguous: row = base + 32 i + lane%32, logical chunk 2 kk + lane/32  -> slot ^ ((row >> 2) & 3)
  // k-slow: 16-lane group b = lane/16, s = lane%16: k = 16 kk + 8 (b/2) + 4 h + s/4,
  //         col = base + 32 j + 16 (b%2) + 4 (s%4); chunk = col/8 ^ 2 (s/4), piece = (s%4)&1
  // k-contiguous: x_fr[kk][0] (blocks add a constant); k-slow: x_fr[h][block] (the swizzle touches the
  // chunk-index bits that the block offset sets, so every 32-column block has its own base address)
  uint32_t a_fr[2][4], b_fr[2][NBK];
  {
    const int b = lane >> 4, s = lane & 15;
    if (!A_NC) {
      const int row = wm * (32 * MB) + (lane & 31);
      for (int kk = 0; kk < 2; ++kk)
        a_fr[kk][0] = a_fr[kk][1] = a_fr[kk][2] = a_fr[kk][3] =
            row * 64 + (((2 * kk + (lane >> 5)) ^ ((lane >> 2) & 3)) * 16);
    } else {
      for (int h = 0; h < 2; ++h)
        for (int blk = 0; blk < 4; ++blk) {
          const int col = wm * 128 + 32 * blk + 16 * (b & 1) + 4 * (s & 3);
          const int k = 8 * (b >> 1) + 4 * h + (s >> 2);
          a_fr[h][blk] = k * 512 + (((col >> 3) ^ (4 * (s >> 2))) * 16) + ((s & 1) * 8);
        }
    }
    if (!B_NC) {
      const int row = wn * (32 * NBK) + (lane & 31);
      for (int kk = 0; kk < 2; ++kk)
        for (int blk = 0; blk < NBK; ++blk)
          b_fr[kk][blk] = DREGION + row * 64 + (((2 * kk + (lane >> 5)) ^ ((lane >> 2) & 3)) * 16);
    } else {
      for (int h = 0; h < 2; ++h)
        for (int blk = 0; blk < NBK; ++blk) {
          const int col = wn * (32 * NBK) + 32 * blk + 16 * (b & 1) + 4 * (s & 3);
          const int k = 8 * (b >> 1) + 4 * h + (s >> 2);
          b_fr[h][blk] = DREGION + k * 512 + (((col >> 3) ^ (4 * (s >> 2))) * 16) + ((s & 1) * 8);
        }
    }
  }
  Frag fa[2][MB], fb[2][NBK];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_AS char*)smem;
  // fragments of k step kk of tile kt go to register set kk; part 0 = the four B fragments,
  // part 1 = A fragments 0,1, part 2 = A fragments 2,3 (so the reads can be spread between MFMAs)
  auto load_frags = [&](int stage, auto kk_tag, int part) {
    constexpr int kk = decltype(kk_tag)::value;
    const uint32_t st = lds0 + (uint32_t)stage * DSTAGE;
    if (part == 0) {
      if (!B_NC) {
        lds_read_kc<0 * 2048>(fb[kk][0], st + b_fr[kk][0]); lds_read_kc<1 * 2048>(fb[kk][1], st + b_fr[kk][0]);
        if (NBK == 4) {
          lds_read_kc<2 * 2048>(fb[kk][NBK - 2], st + b_fr[kk][0]); lds_read_kc<3 * 2048>(fb[kk][NBK - 1], st + b_fr[kk][0]);
        }
      } else {
        lds_read_nc<kk * 8192>(fb[kk][0], st + b_fr[0][0], st + b_fr[1][0]);
        lds_read_nc<kk * 8192>(fb[kk][1], st + b_fr[0][1], st + b_fr[1][1]);
        if (NBK == 4) {
          lds_read_nc<kk * 8192>(fb[kk][NBK - 2], st + b_fr[0][NBK - 2], st + b_fr[1][NBK - 2]);
          lds_read_nc<kk * 8192>(fb[kk][NBK - 1], st + b_fr[0][NBK - 1], st + b_fr[1][NBK - 1]);
        }
      }
    } else if (part == 1) {
      if (!A_NC) {
        lds_read_kc<0 * 2048>(fa[kk][0], st + a_fr[kk][0]); lds_read_kc<1 * 2048>(fa[kk][1], st + a_fr[kk][0]);
      } else {
        lds_read_nc<kk * 8192>(fa[kk][0], st + a_fr[0][0], st + a_fr[1][0]);
        lds_read_nc<kk * 8192>(fa[kk][1], st + a_fr[0][1], st + a_fr[1][1]);
      }
    } else {
      if (!A_NC) {
        lds_read_kc<2 * 2048>(fa[kk][2], st + a_fr[kk][0]);
        if (MB == 4) lds_read_kc<3 * 2048>(fa[kk][MB - 1], st + a_fr[kk][0]);
      } else {
        lds_read_nc<kk * 8192>(fa[kk][2], st + a_fr[0][2], st + a_fr[1][2]);
        lds_read_nc<kk * 8192>(fa[kk][MB - 1], st + a_fr[0][3], st + a_fr[1][3]);
      }
    }
  };
  auto frags_ready = [&](int set) {
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
#pragma unroll
    for (int i = 0; i < MB; ++i) ready(fa[set][i]);
#pragma unroll
    for (int j = 0; j < NBK; ++j) ready(fb[set][j]);
  };
  using K0 = std::integral_constant<int, 0>;
  using K1 = std::integral_constant<int, 1>;

  f32x16_t acc[MB][NBK];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NBK; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  if (GATHER) {
    int g_pro[4][4];
#pragma unroll
    for (int t4 = 0; t4 < 4; ++t4) gather_fetch(t4, g_pro[t4]);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
#pragma unroll
    for (int t4 = 0; t4 < 4; ++t4) {
      gather_rows(g_pro[t4]);
      request_half(t4, 0);
      if (t4 < 3) request_half(t4, 1);
    }
  } else {
    request_half(0, 0); request_half(0, 1);
    request_half(1, 0); request_half(1, 1);
    request_half(2, 0); request_half(2, 1);
    request_half(3, 0);
  }
  // The padding test comes after the first requests are on their way, so that reading the counts
  // delays no tile that has work (a padding tile has fetched a few zeros for nothing).
  if (KIND != KIND_TN && p.cnt != nullptr) {
    const int r_end = min(m0 + TMR, p.Mdim);
    bool pad = true;
    for (int sc = m0 / p.Cc; sc * p.Cc < r_end; ++sc) {
      const int c_lo = max(m0 - sc * p.Cc, 0);
      if (c_lo < p.cnt[sc * p.G + g]) { pad = false; break; }
    }
    if (pad) {
      __builtin_amdgcn_s_waitcnt(0x0070);   // the requests in flight write LDS: let them land before leaving
      f32x16_t none[MB][NBK] = {};
      store_tile_lds<KIND, EPI, MB, NBK>(p, none, smem, g, m0 + wm * (32 * MB), n0 + wn * (32 * NBK), lane, true);
      return;
    }
  }
  // this wave's requests for tile 0 have landed (the 5 RPW issued after them may be in flight)
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(5 * RPW));
  __builtin_amdgcn_s_barrier();
  load_frags(0, K0{}, 0); load_frags(0, K0{}, 1); load_frags(0, K0{}, 2);

  auto mfma_row = [&](int set, int i) {
#pragma unroll
    for (int j = 0; j < NBK; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j].v, fa[set][i].v, acc[i][j], 0, 0, 0);
  };
  auto next_stage = [](int s_) { return s_ + 1 == DSTAGES ? 0 : s_ + 1; };
  // Each k tile is two MFMA steps of MB rows (NBK MFMAs each).  Between the rows go, one piece at
  // a time, the fragment reads of the next step and the tile requests, so that neither the LDS nor
  // the address path sees a burst and the matrix pipe always has work queued.
  //   step 0: B-operand requests of tile kt+3;  step 1: barrier, then A-operand requests of tile kt+4
  // (stage of tile t = t mod 5: s0 holds tile kt, s1 tile kt+1, s3 tile kt+3, s4 tile kt+4 = the stage of kt-1)
  int s0 = 0, s1 = 1, s3 = 3, s4 = 4;
  for (int kt = 0; kt < nk; ++kt) {
    frags_ready(0);
    int g_idx[4];
    if (GATHER) gather_fetch(kt + 4, g_idx);   // arrives by frags_ready(1)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      mfma_row(0, i);
      __builtin_amdgcn_sched_barrier(0);
      if (i < 3) load_frags(s0, K1{}, i);
      if (i < RPW) request1(kt + 3, s3, 1, i);
      __builtin_amdgcn_sched_barrier(0);
    }
    frags_ready(1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_row(1, 0);
    __builtin_amdgcn_sched_barrier(0);
    // tile kt+1 has landed (the 4 RPW requests of tiles kt+2, kt+3 issued after it may still be in flight)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(4 * RPW));
    __builtin_amdgcn_s_barrier();        // everyone is past tile kt-1, and tile kt+1 is complete
    __builtin_amdgcn_sched_barrier(0);
    if (GATHER) gather_rows(g_idx);    // rows of tile kt+4
#pragma unroll
    for (int i = 1; i < MB; ++i) {
      load_frags(s1, K0{}, i - 1);
      if (MB == 3 && i == 2) load_frags(s1, K0{}, 2);
      if (i - 1 < RPW) request1(kt + 4, s4, 0, i - 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_row(1, i);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (RPW == 4) request1(kt + 4, s4, 0, 3);
    s0 = s1; s1 = next_stage(s1); s3 = next_stage(s3); s4 = next_stage(s4);
  }
  __builtin_amdgcn_s_waitcnt(0x0070);  // drain trailing (empty) requests and fragment reads before LDS is released

  __syncthreads();  // every wave is done reading fragments: the stage memory can be reused
  store_tile_lds<KIND, EPI, MB, NBK>(p, acc, smem + wave * (DSTAGES * DSTAGE / (2 * WN)), g, m0 + wm * (32 * MB),
                                 n0 + wn * (32 * NBK), lane);
}

template <int KIND, int EPI, int WN, int TMR = 256, bool GATHER = false>
__global__ __launch_bounds__(128 * WN) void ffn_gemm_dma(const GemmArgs p) {
  __shared__ __attribute__((aligned(1024))) char smem[DSTAGES * DSTAGE];
  gemm_dma_tile<KIND, EPI, WN, TMR, GATHER>(p, smem, (int)blockIdx.x);
}

// The three GEMMs of the backward pass that only depend on dZ, in one launch: dX = dZ W1^T (row-tiled,
// the long tiles, first in the grid) and the two weight gradients.  nbx and nbw are the (multiple-of-8)
// workgroup counts of the first two problems.
template <int TMR_X, bool GATHER_W1 = false>   // GATHER_W1: the third problem reads its A operand through a slot map
__global__ __launch_bounds__(512) void ffn_bwd_trio(const GemmArgs px, const GemmArgs pw2, const GemmArgs pw1, int nbx,
                                                    int nbw) {
  __shared__ __attribute__((aligned(1024))) char smem[DSTAGES * DSTAGE];
  const int b = (int)blockIdx.x;
  if (b < nbx) gemm_dma_tile<KIND_NT, EPI_STORE, 4, TMR_X>(px, smem, b);
  else if (b < nbx + nbw) gemm_dma_tile<KIND_TN, EPI_STORE, 4, 256>(pw2, smem, b - nbx);
  else gemm_dma_tile<KIND_TN, EPI_STORE, 4, 256, GATHER_W1>(pw1, smem, b - nbx - nbw);
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
          if (KIND == KIND_TN) {
            const int64_t row = a_src_row(p, k0 + k, g);
            if (row >= 0) v = A[row * p.lda + m0 + i];
          }
          else {
            const int64_t row = a_src_row(p, m0 + i, g);
            if (row >= 0) v = A[row * p.lda + k0 + k];
          }
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
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
int num_cus() {
  static int n = 0;   // same on every device of a node
  if (n == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n = v;
    else n = 256;
  }
  return n;
}

// Which bf16 kernel and tile a grouped GEMM gets: tile_m x tile_n output tiles; dma = the LDS-DMA
// kernel (the only one that skips padding rows).  `tile` is the caller's hint (MOE_TILE_*).
struct TilePlan {
  bool dma;
  int tile_m, tile_n;
};
TilePlan plan_tiles(int tile, bool tn, int G, int Mdim, int Ndim) {
  TilePlan t;
  const int64_t big_tiles = (int64_t)G * ((Mdim + 255) / 256) * ((Ndim + 255) / 256);
  t.dma = tile == MOE_TILE_AUTO ? big_tiles >= 64 : tile != MOE_TILE_SMALL;
  t.tile_n = t.dma ? 256 : 128;
  t.tile_m = t.tile_n;
  // 192-row tiles when they need no more rounds of the chip's compute units (weighted by tile height)
  if (t.dma && !tn && tile != MOE_TILE_256) {
    const int64_t tiles_n = (Ndim + 255) / 256;
    const int64_t t256 = (int64_t)G * ((Mdim + 255) / 256) * tiles_n;
    const int64_t t192 = (int64_t)G * ((Mdim + 191) / 192) * tiles_n;
    const int64_t cu = num_cus();
    if (tile == MOE_TILE_192 || ((t192 + cu - 1) / cu) * 192 <= ((t256 + cu - 1) / cu) * 256) t.tile_m = 192;
  }
  return t;
}

// fills the tile counts and buffer sizes of a bf16 problem
TilePlan prepare_bf16(GemmArgs& a, bool tn, int tile) {
  a.kchunks = (a.Cc + KT - 1) / KT;
  const uint64_t act_rows = (uint64_t)a.n_src * a.G * a.Cc;
  a.a_bytes = (a.gather ? (uint64_t)a.gather_rows : act_rows) * (uint64_t)a.lda * 2;
  a.b_bytes = tn ? act_rows * (uint64_t)a.ldb * 2 : (uint64_t)a.G * (uint64_t)a.b_goff * 2;
  const TilePlan t = plan_tiles(tile, tn, a.G, a.Mdim, a.Ndim);
  a.tiles_n = (a.Ndim + t.tile_n - 1) / t.tile_n;
  a.tiles_m = (a.Mdim + t.tile_m - 1) / t.tile_m;
  a.total_tiles = a.G * a.tiles_m * a.tiles_n;
  return t;
}

template <int KIND, int EPI>
void launch_gemm(GemmArgs a, int dtype, int tile, hipStream_t st) {
  if (dtype == MOE_F32) {
    a.tiles_m = (a.Mdim + 63) / 64;
    a.tiles_n = (a.Ndim + 63) / 64;
    a.total_tiles = a.G * a.tiles_m * a.tiles_n;
    hipLaunchKernelGGL((ffn_gemm_f32<KIND, EPI>), dim3(a.total_tiles), dim3(256), 0, st, a);
    return;
  }
  const TilePlan t = prepare_bf16(a, KIND == KIND_TN, tile);
  const dim3 grid((unsigned)(((a.total_tiles + 7) / 8) * 8));
  if (!t.dma) {
    hipLaunchKernelGGL((ffn_gemm_bf16<128, 128, 2, 2, KIND, EPI>), grid, dim3(256), 0, st, a);
  } else if (t.tile_m == 192) {
    if constexpr (KIND != KIND_TN) hipLaunchKernelGGL((ffn_gemm_dma<KIND, EPI, 4, 192>), grid, dim3(512), 0, st, a);
  } else if (KIND == KIND_TN && a.gather != nullptr) {
    if constexpr (KIND == KIND_TN) hipLaunchKernelGGL((ffn_gemm_dma<KIND, EPI, 4, 256, true>), grid, dim3(512), 0, st, a);
  } else {
    hipLaunchKernelGGL((ffn_gemm_dma<KIND, EPI, 4>), grid, dim3(512), 0, st, a);
  }
}

inline bool valid_tile(int tile) { return tile >= MOE_TILE_AUTO && tile <= MOE_TILE_192; }

int check_ffn_shape(int dtype, int n_src, int G, int64_t C, int M, int H, int esp_idx, int n_esp) {
  MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_EINVAL);
  MOE_REQUIRE(n_src >= 1 && G >= 1 && C >= 1 && M >= 1 && H >= 1, MOE_EINVAL);
  MOE_REQUIRE(n_esp >= 1 && esp_idx >= 0 && esp_idx < n_esp && H % n_esp == 0, MOE_EINVAL);
  const int Hl = H / n_esp;
  MOE_REQUIRE(M % 8 == 0 && Hl % 8 == 0, MOE_EUNSUPPORTED);
  MOE_REQUIRE((int64_t)n_src * C < (1ll << 31) && (int64_t)n_src * G * C < (1ll << 31), MOE_EUNSUPPORTED);
  if (dtype == MOE_BF16) {  // 32-bit byte offsets inside one activation tensor / one expert's weight matrix
    const uint64_t wide = (uint64_t)(M > Hl ? M : Hl);
    MOE_REQUIRE((uint64_t)n_src * G * C * wide * 2 <= 0xFFFFFFF0ull, MOE_EUNSUPPORTED);
    MOE_REQUIRE((uint64_t)M * H * 2 <= 0xFFFFFFF0ull, MOE_EUNSUPPORTED);
  }
  return MOE_OK;
}

}  // namespace

// multiplied rows of a row-tiled GEMM (outputs [R rows per expert] x N), or of the reduction of a
// weight-gradient GEMM, given host-side row counts
static double rows_multiplied(int tile, bool tn, int dtype, int n_src, int G, int64_t C, int Mdim, int Ndim,
                              const int32_t* cnt) {
  const int64_t R = (int64_t)n_src * C;
  const TilePlan t = plan_tiles(tile, tn, G, Mdim, Ndim);
  if (cnt == nullptr || dtype != MOE_BF16 || !t.dma) return (double)G * (double)R;
  double rows = 0;
  for (int g = 0; g < G; ++g) {
    if (tn) {
      if (n_src != 1) { rows += (double)R; continue; }
      const int64_t c = cnt[g] < 0 ? 0 : cnt[g];
      rows += (double)(c < C ? c : C);
    } else {
      for (int64_t m0 = 0; m0 < R; m0 += t.tile_m) {
        const int64_t r_end = m0 + t.tile_m < R ? m0 + t.tile_m : R;
        bool pad = true;
        for (int64_t sc = m0 / C; sc * C < r_end; ++sc) {
          const int64_t c_lo = m0 - sc * C > 0 ? m0 - sc * C : 0;
          if (c_lo < cnt[sc * G + g]) { pad = false; break; }
        }
        if (!pad) rows += (double)(r_end - m0);
      }
    }
  }
  return rows;
}

extern "C" double moe_ffn_executed_flops(int dtype, int n_src, int G, int64_t C, int M, int H, int n_esp,
                                         const int32_t* row_counts_host, int tile, int backward) {
  if (check_ffn_shape(dtype, n_src, G, C, M, H, 0, n_esp) != MOE_OK || !valid_tile(tile)) return 0.0;
  const int Hl = H / n_esp;
  const int R = (int)(n_src * C);
  const int32_t* c = row_counts_host;
  const double mh = 2.0 * (double)M * (double)Hl;
  if (!backward)   // Z = X W1 (rows x Hl), Y = A W2 (rows x M)
    return mh * (rows_multiplied(tile, false, dtype, n_src, G, C, R, Hl, c) + rows_multiplied(tile, false, dtype, n_src, G, C, R, M, c));
  // dA = dY W2^T (rows x Hl), dW2 (Hl x M over the rows), dW1 (M x Hl over the rows), dX = dZ W1^T (rows x M)
  return mh * (rows_multiplied(tile, false, dtype, n_src, G, C, R, Hl, c) + rows_multiplied(tile, true, dtype, n_src, G, C, Hl, M, c) +
               rows_multiplied(tile, true, dtype, n_src, G, C, M, Hl, c) + rows_multiplied(tile, false, dtype, n_src, G, C, R, M, c));
}

extern "C" size_t moe_ffn_workspace_bytes(int dtype, int n_src, int G, int64_t C, int M, int H, int n_esp) {
  if (check_ffn_shape(dtype, n_src, G, C, M, H, 0, n_esp) != MOE_OK) return 0;
  const size_t esz = dtype == MOE_BF16 ? 2 : 4;
  return moe::align_up((size_t)n_src * G * C * (size_t)(H / n_esp) * esz, 256);   // dZ
}

static int ffn_fwd_impl(const void* X, const int32_t* gather, int gather_k, int64_t gather_rows, int dtype,
                        const void* W1, const void* W2, int n_src, int G, int64_t C, int M, int H, int esp_idx,
                        int n_esp, const int32_t* row_counts, int tile, void* Z, void* A, void* Y, void* stream) {
  if (int rc = check_ffn_shape(dtype, n_src, G, C, M, H, esp_idx, n_esp)) return rc;
  MOE_REQUIRE(valid_tile(tile), MOE_EINVAL);
  MOE_REQUIRE_PTR(X); MOE_REQUIRE_PTR(W1); MOE_REQUIRE_PTR(W2); MOE_REQUIRE_PTR(Z); MOE_REQUIRE_PTR(A);
  MOE_REQUIRE_PTR(Y);
  MOE_REQUIRE((((uintptr_t)row_counts) & 3u) == 0, MOE_EALIGN);
  hipStream_t st = (hipStream_t)stream;
  const int Hl = H / n_esp;
  const int64_t h0 = (int64_t)esp_idx * Hl;

  GemmArgs a{};
  a.G = G; a.n_src = n_src; a.Cc = (int)C; a.R = (int)(n_src * C); a.cnt = row_counts;
  // Z = X * W1[:, h0:h0+Hl] ; A = GeLU(Z)
  a.A = X; a.lda = M;
  a.gather = gather; a.gather_k = gather_k; a.gather_rows = gather_rows;
  a.B = W1; a.ldb = H; a.b_goff = (int64_t)M * H; a.b_off = h0;
  a.C = Z; a.C2 = A; a.ldc = Hl;
  a.Mdim = a.R; a.Ndim = Hl; a.Kdim = M;
  launch_gemm<KIND_NN, EPI_GELU>(a, dtype, tile, st);
  // Y = A * W2[h0:h0+Hl, :]
  a.A = A; a.lda = Hl;
  a.gather = nullptr; a.gather_k = 0; a.gather_rows = 0;
  a.B = W2; a.ldb = M; a.b_goff = (int64_t)H * M; a.b_off = h0 * M;
  a.C = Y; a.C2 = nullptr; a.ldc = M;
  a.Mdim = a.R; a.Ndim = M; a.Kdim = Hl;
  launch_gemm<KIND_NN, EPI_STORE>(a, dtype, tile, st);
  return moe::check_launch();
}

extern "C" int moe_expert_ffn_fwd(const void* X, int dtype, const void* W1, const void* W2, int n_src, int G,
                                  int64_t C, int M, int H, int esp_idx, int n_esp, const int32_t* row_counts, int tile,
                                  void* Z, void* A, void* Y, void* stream) {
  return ffn_fwd_impl(X, nullptr, 0, 0, dtype, W1, W2, n_src, G, C, M, H, esp_idx, n_esp, row_counts, tile, Z, A, Y, stream);
}

// arguments of the fused-dispatch entry points: token matrix [S, M] and the inverse slot map
static int check_gather(const void* x, int dtype, int64_t S, const int32_t* inv, int k, int M) {
  MOE_REQUIRE(S >= 1 && k >= 1 && k <= MOE_MAX_K, MOE_EINVAL);
  MOE_REQUIRE_PTR(x); MOE_REQUIRE_PTR(inv);
  MOE_REQUIRE((int64_t)S * k <= (1ll << 29), MOE_EUNSUPPORTED);   // slot entries t k + j are divided by multiplication
  if (dtype == MOE_BF16) MOE_REQUIRE((uint64_t)S * (uint64_t)M * 2 <= 0xFFFFFFF0ull, MOE_EUNSUPPORTED);
  return MOE_OK;
}

extern "C" int moe_expert_ffn_fwd_gather(const void* x, int dtype, int64_t S, const int32_t* inv, int k, const void* W1,
                                         const void* W2, int E, int64_t C, int M, int H, int esp_idx, int n_esp,
                                         const int32_t* row_counts, int tile, void* Z, void* A, void* Y, void* stream) {
  if (int rc = check_gather(x, dtype, S, inv, k, M)) return rc;
  return ffn_fwd_impl(x, inv, k, S, dtype, W1, W2, 1, E, C, M, H, esp_idx, n_esp, row_counts, tile, Z, A, Y, stream);
}

static int ffn_bwd_impl(const void* dY, const void* X, const int32_t* gather, int gather_k, int64_t gather_rows,
                        const void* Z, const void* A, const void* W1, const void* W2, int dtype, int n_src, int G,
                        int64_t C, int M, int H, int esp_idx, int n_esp, const int32_t* row_counts, int tile, void* dX,
                        void* dW1, void* dW2, void* ws, size_t ws_bytes, void* stream) {
  if (int rc = check_ffn_shape(dtype, n_src, G, C, M, H, esp_idx, n_esp)) return rc;
  MOE_REQUIRE(valid_tile(tile), MOE_EINVAL);
  MOE_REQUIRE_PTR(dY); MOE_REQUIRE_PTR(X); MOE_REQUIRE_PTR(Z); MOE_REQUIRE_PTR(A); MOE_REQUIRE_PTR(W1);
  MOE_REQUIRE_PTR(W2); MOE_REQUIRE_PTR(dX); MOE_REQUIRE_PTR(dW1); MOE_REQUIRE_PTR(dW2);
  const size_t need = moe_ffn_workspace_bytes(dtype, n_src, G, C, M, H, n_esp);
  MOE_REQUIRE(ws != nullptr && ws_bytes >= need, MOE_EWORKSPACE);
  MOE_REQUIRE(moe::aligned16(ws), MOE_EALIGN);
  MOE_REQUIRE((((uintptr_t)row_counts) & 3u) == 0, MOE_EALIGN);
  hipStream_t st = (hipStream_t)stream;
  const int Hl = H / n_esp;
  const int64_t h0 = (int64_t)esp_idx * Hl;
  const void* Act = A;
  void* dZ = ws;

  GemmArgs a{};
  a.G = G; a.n_src = n_src; a.Cc = (int)C; a.R = (int)(n_src * C); a.cnt = row_counts;
  // dA = dY * W2[h0:h0+Hl, :]^T ; dZ = dA * GeLU'(Z)
  a.A = dY; a.lda = M;
  a.B = W2; a.ldb = M; a.b_goff = (int64_t)H * M; a.b_off = h0 * M;
  a.C = dZ; a.C2 = nullptr; a.Zin = Z; a.ldc = Hl;
  a.Mdim = a.R; a.Ndim = Hl; a.Kdim = M;
  launch_gemm<KIND_NT, EPI_DGELU>(a, dtype, tile, st);
  // dW2[h0:h0+Hl, :] = Act^T * dY
  GemmArgs w2 = a;
  w2.A = Act; w2.lda = Hl;
  w2.B = dY; w2.ldb = M;
  w2.C = dW2; w2.C2 = nullptr; w2.Zin = nullptr; w2.ldc = M; w2.c_goff = (int64_t)H * M; w2.c_off = h0 * M;
  w2.Mdim = Hl; w2.Ndim = M; w2.Kdim = a.R;
  // dW1[:, h0:h0+Hl] = X^T * dZ
  GemmArgs w1 = w2;
  w1.A = X; w1.lda = M;
  w1.gather = gather; w1.gather_k = gather_k; w1.gather_rows = gather_rows;
  w1.gather_magic = gather_k > 1 ? (uint32_t)((0x100000000ull + (uint64_t)gather_k - 1) / (uint64_t)gather_k) : 0u;
  w1.B = dZ; w1.ldb = Hl;
  w1.C = dW1; w1.ldc = H; w1.c_goff = (int64_t)M * H; w1.c_off = h0;
  w1.Mdim = M; w1.Ndim = Hl; w1.Kdim = a.R;
  // dX = dZ * W1[:, h0:h0+Hl]^T
  GemmArgs dx = w1;
  dx.A = dZ; dx.lda = Hl;
  dx.gather = nullptr; dx.gather_k = 0; dx.gather_rows = 0; dx.gather_magic = 0;
  dx.B = W1; dx.ldb = H; dx.b_goff = (int64_t)M * H; dx.b_off = h0;
  dx.C = dX; dx.ldc = M; dx.c_goff = 0; dx.c_off = 0;
  dx.Mdim = a.R; dx.Ndim = M; dx.Kdim = Hl;
  if (dtype == MOE_BF16) {
    // the three are independent: one launch, long row tiles first, if all of them take the LDS-DMA kernel
    GemmArgs px = dx, p2 = w2, p1 = w1;
    const TilePlan tx = prepare_bf16(px, false, tile), t2 = prepare_bf16(p2, true, tile), t1 = prepare_bf16(p1, true, tile);
    if (tx.dma && t2.dma && t1.dma) {
      const int nbx = (px.total_tiles + 7) / 8 * 8, nb2 = (p2.total_tiles + 7) / 8 * 8, nb1 = (p1.total_tiles + 7) / 8 * 8;
      const dim3 grid((unsigned)(nbx + nb2 + nb1));
      if (gather) {
        if (tx.tile_m == 192) hipLaunchKernelGGL((ffn_bwd_trio<192, true>), grid, dim3(512), 0, st, px, p2, p1, nbx, nb2);
        else hipLaunchKernelGGL((ffn_bwd_trio<256, true>), grid, dim3(512), 0, st, px, p2, p1, nbx, nb2);
      } else {
        if (tx.tile_m == 192) hipLaunchKernelGGL((ffn_bwd_trio<192>), grid, dim3(512), 0, st, px, p2, p1, nbx, nb2);
        else hipLaunchKernelGGL((ffn_bwd_trio<256>), grid, dim3(512), 0, st, px, p2, p1, nbx, nb2);
      }
      return moe::check_launch();
    }
  }
  launch_gemm<KIND_TN, EPI_STORE>(w2, dtype, tile, st);
  launch_gemm<KIND_TN, EPI_STORE>(w1, dtype, tile, st);
  launch_gemm<KIND_NT, EPI_STORE>(dx, dtype, tile, st);
  return moe::check_launch();
}

extern "C" int moe_expert_ffn_bwd(const void* dY, const void* X, const void* Z, const void* A, const void* W1,
                                  const void* W2, int dtype, int n_src, int G, int64_t C, int M, int H, int esp_idx,
                                  int n_esp, const int32_t* row_counts, int tile, void* dX, void* dW1, void* dW2,
                                  void* ws, size_t ws_bytes, void* stream) {
  return ffn_bwd_impl(dY, X, nullptr, 0, 0, Z, A, W1, W2, dtype, n_src, G, C, M, H, esp_idx, n_esp, row_counts, tile, dX,
                      dW1, dW2, ws, ws_bytes, stream);
}

extern "C" int moe_expert_ffn_bwd_gather(const void* dY, const void* x, int64_t S, const int32_t* inv, int k,
                                         const void* Z, const void* A, const void* W1, const void* W2, int dtype, int E,
                                         int64_t C, int M, int H, int esp_idx, int n_esp, const int32_t* row_counts,
                                         int tile, void* dX, void* dW1, void* dW2, void* ws, size_t ws_bytes,
                                         void* stream) {
  if (int rc = check_gather(x, dtype, S, inv, k, M)) return rc;
  MOE_REQUIRE((int64_t)E * C <= (1ll << 29), MOE_EUNSUPPORTED);   // 32-bit byte offsets into the slot map
  return ffn_bwd_impl(dY, x, inv, k, S, Z, A, W1, W2, dtype, 1, E, C, M, H, esp_idx, n_esp, row_counts, tile, dX, dW1, dW2,
                      ws, ws_bytes, stream);
}
