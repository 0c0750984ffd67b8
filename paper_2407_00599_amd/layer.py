"""Call sequence of one rank's MoE layer over the C ABI, with preallocated device buffers.

`MoERankLayer` strings the entry points together the way a training step would between the
collectives of Section III (gate -> dispatch -> [AlltoAll] -> expert FFN -> [AlltoAll] ->
combine, and the mirror image backward).  With all E experts local and the N_ESP shards run
one after the other on the same GPU it evaluates the whole layer ("closed world"), which is
what the parity tests compare with the CPU checker.  Nothing of the method is computed here: every
step is a library call and torch only owns the memory (MoERankShape.fill_stand_ins copies buffers where a
collective would move them).
"""
from __future__ import annotations

import torch

from . import api


class MoERankLayer:
    def __init__(self, S_total, M, H, E, k, f, dtype=torch.bfloat16, n_mp=1, mp_idx=0, n_esp=1,
                 norm_topk=-1, device="cuda:0"):
        self.S_total, self.M, self.H, self.E, self.k, self.f = S_total, M, H, E, k, f
        self.n_mp, self.mp_idx, self.n_esp, self.norm_topk = n_mp, mp_idx, n_esp, norm_topk
        self.dtype, self.dev = dtype, torch.device(device)
        self.S = S = S_total // n_mp
        self.C = C = api.moe_capacity(S, E, k, f)
        self.Hl = Hl = H // n_esp
        self.dt = api.MOE_BF16 if dtype == torch.bfloat16 else api.MOE_F32
        dev = self.dev
        i32, f32 = torch.int32, torch.float32
        e = lambda *shape, dt=dtype: torch.empty(shape, dtype=dt, device=dev)
        self.logits = e(S, E, dt=f32); self.idx = e(S, k, dt=i32); self.slot = e(S, k, dt=i32)
        self.w = e(S, k, dt=f32); self.inv = e(E, C, dt=i32); self.counts = e(E, dt=i32)
        self.buf = e(E, C, M)
        self.Z = e(n_esp, E, C, Hl); self.A = e(n_esp, E, C, Hl)
        self.Yret = e(n_esp, E, C, M)
        self.y = e(S, M)
        # backward
        self.dYret = e(E, C, M); self.dw = e(S, k, dt=f32)
        self.dbuf = e(n_esp, E, C, M)
        self.dW1 = e(E, M, H); self.dW2 = e(E, H, M)
        self.dx = e(S, M); self.dlogits = e(S, E, dt=f32); self.dWg = e(M, E, dt=f32); self.dbias = e(E, dt=f32)
        nbytes = max(api.moe_gate_workspace_bytes(S, E, k),
                     api.moe_ffn_workspace_bytes(self.dt, 1, E, C, M, H, n_esp),
                     api.moe_gate_bwd_workspace_bytes(S, M, E), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def gate(self, x_full, Wg, bias):
        api.moe_gate_topk(x_full, Wg, bias, self.S_total, self.M, self.E, self.k, self.C, self.mp_idx, self.n_mp,
                          self.norm_topk, self.logits, self.idx, self.slot, self.w, self.inv, self.counts, self.ws)

    def forward(self, x_full, Wg, bias, W1, W2):
        """x_full [S_total, M]; returns y [S, M] for the rank's token block."""
        S, M, E, k, C, H = self.S, self.M, self.E, self.k, self.C, self.H
        self.x = x_full[self.mp_idx * S:(self.mp_idx + 1) * S]
        self.Wg, self.W1, self.W2 = Wg, W1, W2
        self.gate(x_full, Wg, bias)
        api.moe_dispatch(self.x, S, M, E, k, C, self.inv, None, self.buf)
        for j in range(self.n_esp):           # the N_ESP shards of every expert, one after the other
            api.moe_expert_ffn_fwd(self.buf, W1, W2, 1, E, C, M, H, j, self.n_esp, self.Z[j], self.A[j], self.Yret[j],
                                   self.counts)
        api.moe_combine_fwd(self.Yret, self.n_esp, S, M, E, k, C, self.idx, self.slot, self.w, self.y)
        return self.y

    def forward_fused_dispatch(self, x_full, Wg, bias, W1, W2):
        """Forward with the dispatch fused into the first GEMM (no [E, C, M] buffer is written);
        backward_fused_dispatch() is its backward."""
        S, M, E, k, C, H = self.S, self.M, self.E, self.k, self.C, self.H
        self.x = x_full[self.mp_idx * S:(self.mp_idx + 1) * S]
        self.Wg, self.W1, self.W2 = Wg, W1, W2
        self.gate(x_full, Wg, bias)
        for j in range(self.n_esp):
            api.moe_expert_ffn_fwd_gather(self.x, self.inv, S, k, W1, W2, E, C, M, H, j, self.n_esp, self.Z[j],
                                          self.A[j], self.Yret[j], self.counts)
        api.moe_combine_fwd(self.Yret, self.n_esp, S, M, E, k, C, self.idx, self.slot, self.w, self.y)
        return self.y

    def backward_fused_dispatch(self, dy):
        """backward() without the dispatched buffer: the weight gradient of the first GEMM gathers its rows."""
        S, M, E, k, C, H = self.S, self.M, self.E, self.k, self.C, self.H
        api.moe_combine_bwd(dy, self.Yret, self.n_esp, S, M, E, k, C, self.idx, self.slot, self.inv, self.w,
                            self.dYret, self.dw)
        for j in range(self.n_esp):
            api.moe_expert_ffn_bwd_gather(self.dYret, self.x, self.inv, S, k, self.Z[j], self.A[j], self.W1, self.W2,
                                          E, C, M, H, j, self.n_esp, self.dbuf[j], self.dW1, self.dW2, self.ws,
                                          self.counts)
        api.moe_combine_fwd(self.dbuf, self.n_esp, S, M, E, k, C, self.idx, self.slot, None, self.dx)
        api.moe_gate_bwd(self.dw, self.w, self.idx, self.logits, self.x, self.Wg, S, M, E, k, self.norm_topk,
                         self.dlogits, self.dWg, self.dbias, self.dx, 1, self.ws)
        return self.dx

    def backward(self, dy):
        S, M, E, k, C, H = self.S, self.M, self.E, self.k, self.C, self.H
        api.moe_combine_bwd(dy, self.Yret, self.n_esp, S, M, E, k, C, self.idx, self.slot, self.inv, self.w,
                            self.dYret, self.dw)
        for j in range(self.n_esp):
            api.moe_expert_ffn_bwd(self.dYret, self.buf, self.Z[j], self.A[j], self.W1, self.W2, 1, E, C, M, H, j,
                                   self.n_esp, self.dbuf[j], self.dW1, self.dW2, self.ws, self.counts)
        # backward of dispatch = unweighted combine of the (n_esp partial) input gradients
        api.moe_combine_fwd(self.dbuf, self.n_esp, S, M, E, k, C, self.idx, self.slot, None, self.dx)
        api.moe_gate_bwd(self.dw, self.w, self.idx, self.logits, self.x, self.Wg, S, M, E, k, self.norm_topk,
                         self.dlogits, self.dWg, self.dbias, self.dx, 1, self.ws)
        return self.dx


class MoERankShape:
    """One rank's step at its real shapes when the experts are NOT all local (N_EP > 1 or
    N_ESP > 1).  The two EP&ESP-AlltoAlls cannot run on one GPU, so the tensors that would
    arrive through them are stand-ins of the right shape (fill_stand_ins builds them from the rank's own data):
        Xrecv  [n_src, G, C, M]    what the first AlltoAll delivers to the local experts
        Yret   [n_esp, E, C, M]    what the second AlltoAll returns (N_ESP partial sums)
        dYrecv [n_src, G, C, M]    backward: gradient rows delivered to the local experts
        dbuf   [n_esp, E, C, M]    backward: input gradients returned to the token owner
    Every kernel of the path still runs once at the rank's shape; only the data crossing the
    collectives is synthetic.  With n_src = 1, G = E, n_esp = 1 the stand-ins alias the real
    buffers and the step is the complete layer."""

    def __init__(self, S_total, M, H, E, k, f, dtype=torch.bfloat16, n_mp=1, mp_idx=0, n_ep=1, n_esp=1,
                 esp_idx=0, norm_topk=-1, device="cuda:0", tile=0):
        self.S_total, self.M, self.H, self.E, self.k, self.f = S_total, M, H, E, k, f
        self.tile = tile
        self.n_mp, self.mp_idx, self.n_ep, self.n_esp, self.esp_idx = n_mp, mp_idx, n_ep, n_esp, esp_idx
        self.norm_topk = norm_topk
        self.S = S = S_total // n_mp
        self.C = C = api.moe_capacity(S, E, k, f)
        self.G = G = E // n_ep
        self.n_src = n_src = n_ep * n_esp
        self.Hl = Hl = H // n_esp
        self.dt = api.MOE_BF16 if dtype == torch.bfloat16 else api.MOE_F32
        self.closed = (n_src == 1)
        dev = torch.device(device)
        i32, f32 = torch.int32, torch.float32
        e = lambda *shape, dt=dtype: torch.empty(shape, dtype=dt, device=dev)
        self.logits = e(S, E, dt=f32); self.idx = e(S, k, dt=i32); self.slot = e(S, k, dt=i32)
        self.w = e(S, k, dt=f32); self.inv = e(E, C, dt=i32); self.counts = e(E, dt=i32)
        self.buf = e(E, C, M)
        self.Z = e(n_src, G, C, Hl); self.A = e(n_src, G, C, Hl)
        self.Yout = e(n_src, G, C, M)
        self.y = e(S, M)
        self.dYret = e(E, C, M); self.dw = e(S, k, dt=f32)
        self.dXout = e(n_src, G, C, M)
        self.dW1 = e(G, M, H); self.dW2 = e(G, H, M)
        self.dx = e(S, M); self.dlogits = e(S, E, dt=f32); self.dWg = e(M, E, dt=f32); self.dbias = e(E, dt=f32)
        if self.closed:
            self.Xrecv, self.Yret, self.dYrecv, self.dbuf = self.buf.view(1, E, C, M), self.Yout, \
                self.dYret.view(1, E, C, M), self.dXout
            self.row_counts = self.counts      # every expert is local: the gate's demand counts name the padding
        else:
            self.Xrecv = e(n_src, G, C, M); self.Yret = e(n_esp, E, C, M)
            self.dYrecv = e(n_src, G, C, M); self.dbuf = e(n_esp, E, C, M)
            self.row_counts = torch.empty(n_src, G, dtype=i32, device=dev)   # occupancy that would arrive with the AlltoAll
        nbytes = max(api.moe_gate_workspace_bytes(S, E, k),
                     api.moe_ffn_workspace_bytes(self.dt, n_src, G, C, M, H, n_esp),
                     api.moe_gate_bwd_workspace_bytes(S, M, E), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def bind(self, x_full, Wg, bias, W1, W2, dy):
        S = self.S
        self.x_full, self.x = x_full, x_full[self.mp_idx * S:(self.mp_idx + 1) * S]
        self.Wg, self.bias, self.W1, self.W2, self.dy = Wg, bias, W1, W2, dy

    def fill_stand_ins(self):
        """Builds, in one pass over the calls, what the collectives would deliver to a rank that does not hold
        every expert, from the rank's own data (the copies stand in for the AlltoAlls; a peer's tokens are
        distributed like the rank's own): source chunk s of the expert input, and of the gradient input, is
        chunk s mod N_EP of the rank's own send buffer, with the gate's demand counts of those experts as its
        occupancy; the returned buffers are the rank's own expert outputs, chunk for chunk."""
        assert not self.closed
        n_ep, G, C, M = self.n_ep, self.G, self.C, self.M
        self.gate(); self.dispatch()
        send, cnt = self.buf.view(n_ep, G, C, M), self.counts.view(n_ep, G)
        for s in range(self.n_src):
            self.Xrecv[s].copy_(send[s % n_ep]); self.row_counts[s].copy_(cnt[s % n_ep])
        self.row_counts.clamp_(max=C)
        self.ffn_fwd()
        self.Yret.copy_(self.Yout.view(self.n_esp, self.E, C, M))
        self.combine(); self.combine_bwd()
        dsend = self.dYret.view(n_ep, G, C, M)
        for s in range(self.n_src):
            self.dYrecv[s].copy_(dsend[s % n_ep])
        self.ffn_bwd()
        self.dbuf.copy_(self.dXout.view(self.n_esp, self.E, C, M))

    # the individual calls, so a benchmark can time them one by one
    def gate(self):
        api.moe_gate_topk(self.x_full, self.Wg, self.bias, self.S_total, self.M, self.E, self.k, self.C, self.mp_idx,
                          self.n_mp, self.norm_topk, self.logits, self.idx, self.slot, self.w, self.inv, self.counts,
                          self.ws)

    def dispatch(self):
        api.moe_dispatch(self.x, self.S, self.M, self.E, self.k, self.C, self.inv, None, self.buf)

    def ffn_fwd(self):
        api.moe_expert_ffn_fwd(self.Xrecv, self.W1, self.W2, self.n_src, self.G, self.C, self.M, self.H, self.esp_idx,
                               self.n_esp, self.Z, self.A, self.Yout, self.row_counts, self.tile)

    def ffn_fwd_gather(self):
        """dispatch + ffn_fwd in one call (every expert local); not one of STEPS."""
        assert self.closed
        api.moe_expert_ffn_fwd_gather(self.x, self.inv, self.S, self.k, self.W1, self.W2, self.E, self.C, self.M,
                                      self.H, self.esp_idx, self.n_esp, self.Z, self.A, self.Yout, self.row_counts,
                                      self.tile)

    def combine(self):
        api.moe_combine_fwd(self.Yret, self.n_esp, self.S, self.M, self.E, self.k, self.C, self.idx, self.slot,
                            self.w, self.y)

    def combine_bwd(self):
        api.moe_combine_bwd(self.dy, self.Yret, self.n_esp, self.S, self.M, self.E, self.k, self.C, self.idx,
                            self.slot, self.inv, self.w, self.dYret, self.dw)

    def ffn_bwd(self):
        api.moe_expert_ffn_bwd(self.dYrecv, self.Xrecv, self.Z, self.A, self.W1, self.W2, self.n_src, self.G, self.C,
                               self.M, self.H, self.esp_idx, self.n_esp, self.dXout, self.dW1, self.dW2, self.ws,
                               self.row_counts, self.tile)

    def ffn_bwd_gather(self):
        """ffn_bwd that reads the rows of X from the token matrix (every expert local); not one of STEPS."""
        assert self.closed
        api.moe_expert_ffn_bwd_gather(self.dYrecv, self.x, self.inv, self.S, self.k, self.Z, self.A, self.W1, self.W2,
                                      self.E, self.C, self.M, self.H, self.esp_idx, self.n_esp, self.dXout, self.dW1,
                                      self.dW2, self.ws, self.row_counts, self.tile)

    def dispatch_bwd(self):
        api.moe_combine_fwd(self.dbuf, self.n_esp, self.S, self.M, self.E, self.k, self.C, self.idx, self.slot, None,
                            self.dx)

    def gate_bwd(self):
        api.moe_gate_bwd(self.dw, self.w, self.idx, self.logits, self.x, self.Wg, self.S, self.M, self.E, self.k,
                         self.norm_topk, self.dlogits, self.dWg, self.dbias if self.bias is not None else None,
                         self.dx, 1, self.ws)

    STEPS = ("gate", "dispatch", "ffn_fwd", "combine", "combine_bwd", "ffn_bwd", "dispatch_bwd", "gate_bwd")
    # every expert local: the dispatch is fused into the expert GEMMs, no [E, C, M] input buffer is written
    STEPS_FUSED = ("gate", "ffn_fwd_gather", "combine", "combine_bwd", "ffn_bwd_gather", "dispatch_bwd", "gate_bwd")

    def step(self, fused=False):
        for name in (self.STEPS_FUSED if fused else self.STEPS):
            getattr(self, name)()
