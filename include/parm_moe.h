/*
 * parm_moe.h -- C ABI of the per-GPU compute of one rank of a Parm MoE layer on MI355X (gfx950).
 *
 * The layer is the one of Section II-A of the Parm paper ("Mixture-of-Experts Layer"): a
 * gating function (one linear layer, softmax, top-k) builds G in R^{E x T x M}, expert i
 * processes G[i,:,:] with two FFN matrices (M,H) and (H,M) around an activation, and the
 * expert outputs are combined back to token order.  Parm (Section III) runs it under
 * MP+EP+ESP: the MP group splits the tokens on entry (PauseMP, schedule S1), the experts are
 * spread over N_EP ranks and each expert's hidden dimension over N_ESP shards, and two
 * EP&ESP-AlltoAlls sit between dispatch / expert FFN / combine.  This library is what ONE
 * rank computes between those collectives, forward and backward.  It performs no
 * communication.
 *
 * Notation (Table 1 of the paper): S tokens gated by this rank (= B*L/N_MP), M embedding
 * size, H expert hidden size, E experts in total, k experts per token, f capacity factor,
 * C = the paper's T, rows per expert.  G = E/N_EP local experts, n_src = N_EP*N_ESP peers
 * that send this rank a [G, C, M] chunk each, H_l = H/N_ESP.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers to dense row-major memory owned by the caller,
 *     16-byte aligned.  The library allocates nothing and keeps no state between calls;
 *     scratch memory is a caller-supplied workspace `ws` of at least the size the matching
 *     *_workspace_bytes() helper returns (ws may be NULL when that size is 0).
 *   - `dtype` is MOE_F32 or MOE_BF16 and names the storage type of activations and expert
 *     weights.  Gate weights, logits, combine weights and their gradients are always fp32,
 *     index tensors int32.  Accumulation is fp32 (fp64 for the gate logits).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream);
 *     no call synchronises with the host.  Outputs are fully overwritten, never accumulated,
 *     unless stated.
 *   - Return value: MOE_OK, or a negative error.  Arguments are validated on the host before
 *     anything is launched; on an error nothing was enqueued.  No exceptions, no aborts, no
 *     output on stdout/stderr.
 *   - MP and ESP are plain integers: (mp_idx, n_mp) picks this rank's block of the token
 *     rows, (esp_idx, n_esp) picks the hidden slice [esp_idx*H/n_esp, (esp_idx+1)*H/n_esp)
 *     of the FULL weight tensors W1 [G,M,H] and W2 [G,H,M].
 *   - Limits: 1 <= k <= 8, k <= E <= 256, M % 8 == 0, H_l % 8 == 0 (both storage types).
 */
#ifndef PARM_MOE_H
#define PARM_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MOE_F32 = 0, MOE_BF16 = 1 };

enum {
  MOE_OK = 0,
  MOE_EINVAL = -1,       /* a shape or argument is out of range / inconsistent */
  MOE_EUNSUPPORTED = -2, /* valid in the paper's terms but outside this build's limits */
  MOE_EALIGN = -3,       /* a pointer is not 16-byte aligned */
  MOE_ELAUNCH = -4,      /* HIP reported an error when enqueuing */
  MOE_EWORKSPACE = -5,   /* ws is NULL or ws_bytes is too small */
  MOE_ENULL = -6,        /* a required pointer is NULL */
  MOE_ESCRATCH = -7      /* the problem needs more scratch than the library's static array holds */
};

/* Human-readable name of an error code (static storage, never NULL). */
const char* moe_strerror(int err);

/* Library ABI version (bumped when a signature changes). */
int moe_abi_version(void);

/* Expert capacity, Section II-A: T := k * f * B * L / E, for the S tokens this rank gates
 * (schedule S1 gates the MP slice, Section III-B).  Rounded up, evaluated in double as
 * ((k*S)*f)/E, at least 1.  Returns -1 on invalid arguments.  Host function. */
int64_t moe_capacity(int64_t S, int E, int k, double f);

/* ---------------------------------------------------------------------------------------
 * Gate: Section II-A "Gating Function" (linear layer, softmax, top-k, capacity T) on the
 * MP slice of Section III-B.
 *
 *   x         [S_total, M] activations (x_dtype), or NULL: then `logits` is an INPUT and M,
 *             x_dtype and Wg are ignored
 *   Wg        [M, E] fp32 gate weight
 *   gate_bias [E] fp32 or NULL, added to the logits
 *   S_total, n_mp, mp_idx: the rank gates rows [mp_idx*S, (mp_idx+1)*S), S = S_total/n_mp
 *   norm_topk 1: weights = softmax over the k selected logits; 0: full-softmax probability
 *             of each selected expert; -1: 1 when k >= 2, else 0
 *   logits    [S, E] fp32, written (or read when x is NULL)
 *   idx       [S, k] int32 out: selected experts, best first; equal logits -> lower index
 *   w         [S, k] fp32 out: combine weights
 *   slot      [S, k] int32 out: row of (t,j) in expert idx[t,j]'s block, -1 if dropped.
 *             Slots are given choice-major (all first choices, then all second choices...)
 *             and in token order within a choice; an expert keeps the first C.
 *   inv       [E, C] int32 out: t*k+j of the occupant of each slot, -1 if empty
 *   counts    [E] int32 out: assignments that asked for each expert (before capacity)
 * --------------------------------------------------------------------------------------- */
size_t moe_gate_workspace_bytes(int64_t S, int E, int k);

int moe_gate_topk(const void* x, int x_dtype, const float* Wg, const float* gate_bias,
                  int64_t S_total, int M, int E, int k, int64_t C,
                  int mp_idx, int n_mp, int norm_topk,
                  float* logits, int32_t* idx, int32_t* slot, float* w,
                  int32_t* inv, int32_t* counts,
                  void* ws, size_t ws_bytes, void* stream);

/* moe_gate_topk for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as moe_gate_topk, minus the
 * workspace: the per-block histograms live in a static device array of MOE_GATE_STATIC_SCRATCH_BYTES that
 * every GPU the library runs on holds until the process ends.  The call allocates nothing and frees nothing
 * (the first call on a device looks the array's address up, once).  A problem whose
 * moe_gate_workspace_bytes(S, E, k) exceeds the array is rejected with MOE_ESCRATCH (the array covers
 * ceil(S / 64) * k * E <= 262144, e.g. 32768 tokens x top-2 x 256 experts).  Nothing in the array has to
 * start at zero (every word a call reads was written by that call), so it needs no clearing; it is shared by
 * all calls on that GPU: calls that overlap in time on one GPU (different streams or threads) race. */
#define MOE_GATE_STATIC_SCRATCH_BYTES (2u << 20)
int moe_gate_topk_static(const void* x, int x_dtype, const float* Wg, const float* gate_bias,
                         int64_t S_total, int M, int E, int k, int64_t C,
                         int mp_idx, int n_mp, int norm_topk,
                         float* logits, int32_t* idx, int32_t* slot, float* w,
                         int32_t* inv, int32_t* counts, void* stream);

/* ---------------------------------------------------------------------------------------
 * Dispatch: Section II-A defines G in R^{E x T x M}, whose slice G[i,:,:] holds the tokens that
 * go to expert i.  buf[e,c,:] = x[t,:] for the occupant (t,j) = inv[e,c], zeros for
 * empty slots; with w != NULL rows are scaled by w[t,j] (fp32 multiply, rounded to dtype).
 * buf [E,C,M] viewed [N_EP, G, C, M] is the send buffer of the EP&ESP-AlltoAll (Section
 * III-C); the "Dump" that duplicates it N_ESP times is an alias of the same memory.
 *   x [S, M] is the rank's own token block (already offset by the caller).
 * --------------------------------------------------------------------------------------- */
int moe_dispatch(const void* x, int dtype, int64_t S, int M, int E, int k, int64_t C,
                 const int32_t* inv, const float* w, void* buf, void* stream);

/* Schedule S2 (Section III-B: MP is paused after the gate and resumed before the combine): the
 * gate runs on all B*L tokens of the MP group (moe_gate_topk with n_mp = 1, so the capacity
 * comes from B*L), and the MP-Split then hands each MP rank one part of the dispatched [E,C,M]
 * buffer.  This call writes only the rank's part, the slots c0 <= c < c1 of every expert:
 *   buf [E, c1-c0, M],  buf[e, c-c0, :] = x[t,:] (times w[t,j]) for (t,j) = inv[e,c], else 0.
 * The part of rank r out of n is c0 = floor(r*C/n), c1 = floor((r+1)*C/n) (the paper fixes no
 * particular split; contiguous slot ranges keep each part a dense [E,*,M] AlltoAll buffer).  The
 * expert FFN then runs with C := c1-c0; after the MP-AllGather the parts form the full
 * [E,C,M] buffer that moe_combine_fwd reads.  With w != NULL this is also the rank's part of
 * the combine backward (dYret).  MOE_EINVAL unless 0 <= c0 < c1 <= C. */
int moe_dispatch_slots(const void* x, int dtype, int64_t S, int M, int E, int k, int64_t C,
                       int64_t c0, int64_t c1, const int32_t* inv, const float* w, void* buf,
                       void* stream);

/* ---------------------------------------------------------------------------------------
 * Expert FFN on one ESP shard: Section II-A "Experts" (weights (M,H) and (H,M) around an
 * activation) with the hidden dimension split as in Y = sum_p W2^(p) f(W1^(p) X) (Section
 * II-B "Model Parallelism", applied to experts by ESP).  f is the exact (erf) GeLU.
 *
 *   X  [n_src, G, C, M]  receive buffer of the EP&ESP-AlltoAll; local expert g owns the
 *                        n_src*C rows X[:, g, :, :]
 *   W1 [G, M, H], W2 [G, H, M]  full tensors; the shard uses columns / rows
 *                        [esp_idx*H_l, (esp_idx+1)*H_l), H_l = H/n_esp
 *   Z  [n_src, G, C, H_l] out: pre-activation X*W1, dtype          } both saved for backward
 *   A  [n_src, G, C, H_l] out: activation GeLU(Z), dtype           } (the caller owns them)
 *   Y  [n_src, G, C, M]   out: A*W2 -- a partial sum when n_esp > 1
 * In bf16 the GeLU and its derivative are evaluated by odd minimax polynomials of the normal CDF
 * (absolute error below 5e-5 resp. 2e-4, under the bf16 rounding of the stored result); fp32
 * uses erff.
 *
 *   row_counts [n_src, G] int32, device, or NULL: the caller's promise that in chunk (s, g) the
 *                        rows c >= min(row_counts[s,g], C) of X (and of dY in backward) are zero,
 *                        i.e. capacity padding (counts from moe_gate_topk qualify when all experts
 *                        are local).  Results are the same as without it -- FFN(0) = 0 and zero rows
 *                        add nothing to the weight gradients -- but row tiles that hold nothing
 *                        else are not multiplied (their outputs are stored as zeros), and with
 *                        n_src = 1 the weight-gradient reductions stop at the count.
 *
 * Backward (chain rule of the above), given dY [n_src,G,C,M] and the saved Z and A:
 *   dX  [n_src, G, C, M]  out
 *   dW1 [G, M, H], dW2 [G, H, M]  FULL tensors; only the shard's columns / rows are written
 *                        (overwritten, dtype, fp32 accumulation over all n_src*C rows)
 * --------------------------------------------------------------------------------------- */
/* Scratch the backward call needs (the gradient of the pre-activation, [n_src,G,C,H_l]); the
 * forward call needs none.  0 for invalid shapes. */
size_t moe_ffn_workspace_bytes(int dtype, int n_src, int G, int64_t C, int M, int H, int n_esp);

/* Tile hint of the bf16 grouped GEMMs, an argument of every expert-FFN call.  It selects among
 * kernels that compute the same products and may change the fp32 summation order, nothing else:
 *   MOE_TILE_AUTO   per GEMM from its tile count (what a caller should pass)
 *   MOE_TILE_SMALL  128 x 128 output tiles, register-staged kernel (what AUTO picks for tiny GEMMs;
 *                   this kernel ignores row_counts)
 *   MOE_TILE_256    256 x 256 tiles, LDS-DMA kernel
 *   MOE_TILE_192    the same kernel with 192-row tiles wherever the operand layout allows (the
 *                   row-tiled GEMMs; AUTO picks it when it fills the chip's compute units better)
 * Other values: MOE_EINVAL.  Ignored for fp32. */
enum { MOE_TILE_AUTO = 0, MOE_TILE_SMALL = 1, MOE_TILE_256 = 2, MOE_TILE_192 = 3 };

/* Floating-point operations the forward (backward = 0: 2 GEMMs) or backward (backward = 1: 4 GEMMs)
 * call multiplies out for this shape and tile hint: 2 * M * H_l per multiplied row
 * and GEMM, where a row counts if it lies in a row tile that is not skipped (row-tiled GEMMs) or
 * below the count (weight-gradient reductions, n_src = 1).  row_counts_host is a HOST copy of the
 * row_counts passed to the calls, or NULL (every row is multiplied).  Pure host arithmetic, used by
 * the benchmark to price the matrix pipes by executed work.  0 for invalid shapes. */
double moe_ffn_executed_flops(int dtype, int n_src, int G, int64_t C, int M, int H, int n_esp,
                              const int32_t* row_counts_host, int tile, int backward);

int moe_expert_ffn_fwd(const void* X, int dtype, const void* W1, const void* W2,
                       int n_src, int G, int64_t C, int M, int H, int esp_idx, int n_esp,
                       const int32_t* row_counts, int tile, void* Z, void* A, void* Y, void* stream);

/* Forward with the dispatch fused into the first GEMM, for a rank that holds every expert
 * (N_EP = 1; the ESP shards may still run one after the other: no AlltoAll between gate and
 * experts; Section III-B notes that
 * the local duplication before the AlltoAll is virtual, and without an AlltoAll the [E,C,M]
 * buffer itself need not exist): row c of expert e of the first GEMM is read straight from the
 * token matrix through the gate's inverse slot map,
 *   X[e, c, :] = x[inv[e, c] / k, :]   (inv[e, c] < 0: an empty slot, a zero row),
 * which is exactly what moe_dispatch would have written, so Z, A and Y are the same values as
 * moe_dispatch followed by moe_expert_ffn_fwd(n_src = 1, G = E) produces.
 *   x    [S, M]      dtype, device, in (token rows)
 *   inv  [E, C]      int32, device, in (from moe_gate_topk: t * k + j, or -1)
 *   the other arguments as in moe_expert_ffn_fwd with n_src = 1, G = E.
 * S * k may not exceed 2^29, and E * C not for the backward (MOE_EUNSUPPORTED).  Errors as above.
 *
 * moe_expert_ffn_bwd_gather is the matching backward: the weight gradient dW1 = X^T dZ reads its
 * rows of X from the token matrix through the same map (the reduction index is the slot), so a
 * training step needs no dispatched [E, C, M] buffer at all.  dX is still the slot-ordered
 * [1, E, C, M] gradient, which moe_combine_fwd(w = NULL) turns into dx.  Same values as
 * moe_expert_ffn_bwd on the dispatched buffer.  Other arguments as in moe_expert_ffn_bwd with
 * n_src = 1, G = E. */
int moe_expert_ffn_fwd_gather(const void* x, int dtype, int64_t S, const int32_t* inv, int k,
                              const void* W1, const void* W2, int E, int64_t C, int M, int H,
                              int esp_idx, int n_esp, const int32_t* row_counts, int tile,
                              void* Z, void* A, void* Y, void* stream);
int moe_expert_ffn_bwd_gather(const void* dY, const void* x, int64_t S, const int32_t* inv, int k,
                              const void* Z, const void* A, const void* W1, const void* W2,
                              int dtype, int E, int64_t C, int M, int H, int esp_idx, int n_esp,
                              const int32_t* row_counts, int tile,
                              void* dX, void* dW1, void* dW2, void* ws, size_t ws_bytes, void* stream);

int moe_expert_ffn_bwd(const void* dY, const void* X, const void* Z, const void* A,
                       const void* W1, const void* W2, int dtype,
                       int n_src, int G, int64_t C, int M, int H, int esp_idx, int n_esp,
                       const int32_t* row_counts, int tile,
                       void* dX, void* dW1, void* dW2, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Combine: Section II-A, the expert outputs [Q_1..Q_E] are combined into the (B,L,M) layer
 * output; Section III-C, the N_ESP partial sums that come back through the second
 * EP&ESP-AlltoAll are first added locally ("local combine").
 *
 *   Yret [n_part, E, C, M]  returned buffer(s); n_part = N_ESP partial sums (1 if summed)
 *   y[t,:] = sum over j with slot[t,j] >= 0 of  w[t,j] * sum_p Yret[p, idx[t,j], slot[t,j], :]
 *   w == NULL means unit weights: that is the backward of moe_dispatch (dx from dbuf).
 *   Rows of tokens whose every choice was dropped are zero.
 *
 * Backward:  dYret [E, C, M] = w[t,j] * dy[t,:] at the occupant's slot, zeros at empty slots
 *            (every partial sum receives this same gradient);
 *            dw[t,j] = < dy[t,:], sum_p Yret[p, idx[t,j], slot[t,j], :] >, 0 if dropped.
 *            dYret may be NULL (only dw is wanted: under S2 the rank's slot range of dYret
 *            comes from moe_dispatch_slots(dy, ..., w, ...)).
 * --------------------------------------------------------------------------------------- */
int moe_combine_fwd(const void* Yret, int dtype, int n_part, int64_t S, int M, int E, int k,
                    int64_t C, const int32_t* idx, const int32_t* slot, const float* w,
                    void* y, void* stream);

int moe_combine_bwd(const void* dy, const void* Yret, int dtype, int n_part,
                    int64_t S, int M, int E, int k, int64_t C,
                    const int32_t* idx, const int32_t* slot, const int32_t* inv, const float* w,
                    void* dYret, float* dw, void* stream);

/* ---------------------------------------------------------------------------------------
 * Gate backward: chain rule through Section II-A's gating function with the selection held
 * fixed.  dw -> dlogits (softmax over the selected k, or full softmax, as norm_topk says),
 * dWg = x^T dlogits, dgate_bias = column sums of dlogits, dx = dlogits Wg^T.
 *
 *   x [S, M] the rank's token block; logits, idx, w as produced by moe_gate_topk
 *   dlogits [S, E] fp32 out; dWg [M, E] fp32 out; dgate_bias [E] fp32 out or NULL
 *   dx [S, M] (x_dtype): overwritten, or with dx_accumulate = 1 read and added to (so the
 *   gate's share lands on top of the dispatch share computed by moe_combine_fwd(w=NULL))
 * --------------------------------------------------------------------------------------- */
size_t moe_gate_bwd_workspace_bytes(int64_t S, int M, int E);

int moe_gate_bwd(const float* dw, const float* w, const int32_t* idx, const float* logits,
                 const void* x, int x_dtype, const float* Wg,
                 int64_t S, int M, int E, int k, int norm_topk,
                 float* dlogits, float* dWg, float* dgate_bias,
                 void* dx, int dx_accumulate, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Schedule selection, Section V.  Host functions, host pointers, no GPU work.
 *
 * moe_alpha_beta_fit: least-squares fit of t = alpha + beta * x to n >= 2 measured (size, time)
 * pairs of a collective (Section V-A, "Performance Models").  MOE_EINVAL if all sizes are equal.
 *
 * moe_choose_schedule: Algorithm 1.  With x = B L M, T = k f B L / E (Section II-A; the listing's
 * extra factor M in T is taken as a slip, y = E T M N_ESP being the element count it goes on to
 * use) and y = E T M N_ESP:
 *     t_D1 = 2 (alpha_a2a + beta_a2a y / N_MP) + alpha_ag_mp + beta_ag_mp x
 *     t_D2 = alpha_a2a + beta_a2a y / N_MP + alpha_o + beta_o y
 * Returns 1 (S1, also on a tie) or 2 (S2), or a negative error code; t_d1 / t_d2 (optional)
 * receive the two times.
 * --------------------------------------------------------------------------------------- */
int moe_alpha_beta_fit(const double* x, const double* t, int n, double* alpha, double* beta);

int moe_choose_schedule(double alpha_ag_mp, double beta_ag_mp, double alpha_a2a, double beta_a2a,
                        double alpha_o, double beta_o, int64_t B, int64_t L, int E, int M, int k,
                        double f, int n_esp, int n_mp, double* t_d1, double* t_d2);

#ifdef __cplusplus
}
#endif
#endif /* PARM_MOE_H */
