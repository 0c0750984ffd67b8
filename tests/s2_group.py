"""Test scaffolding for schedule S2 (Section III-B): one MP group strung together on one GPU.

The library calls are the product's; the torch copies, zero fills and additions between them stand in for
what the MP-AllGather and the gradient reduction over the MP group would do, which is why this class lives
with the tests and not in the package."""
import torch

from paper_2407_00599_amd import api


class MoES2Group:
    """Schedule S2 (Section III-B) for one MP group, evaluated on one GPU: the gate and the combine see
    all tokens of the group; between them each of the n_mp ranks dispatches, and feeds to the experts,
    only its slot range of the [E, C, M] buffer (moe_dispatch_slots).  The ranks run one after the
    other; the copies of their parts into the full buffers stand in for the MP-AllGather (forward and
    backward), the sum of their weight gradients for the gradient reduction over the group.  All experts
    are local and the N_ESP shards run in turn, as in MoERankLayer."""

    def __init__(self, S_total, M, H, E, k, f, dtype=torch.bfloat16, n_mp=2, n_esp=1, norm_topk=-1, device="cuda:0"):
        self.S, self.M, self.H, self.E, self.k, self.f = S_total, M, H, E, k, f
        self.n_mp, self.n_esp, self.norm_topk = n_mp, n_esp, norm_topk
        S = S_total
        self.C = C = api.moe_capacity(S, E, k, f)
        self.Hl = Hl = H // n_esp
        self.dt = api.MOE_BF16 if dtype == torch.bfloat16 else api.MOE_F32
        self.ranges = [((r * C) // n_mp, ((r + 1) * C) // n_mp) for r in range(n_mp)]
        dev = torch.device(device)
        i32, f32 = torch.int32, torch.float32
        e = lambda *shape, dt=dtype: torch.empty(shape, dtype=dt, device=dev)
        self.logits = e(S, E, dt=f32); self.idx = e(S, k, dt=i32); self.slot = e(S, k, dt=i32)
        self.w = e(S, k, dt=f32); self.inv = e(E, C, dt=i32); self.counts = e(E, dt=i32)
        self.parts = [e(E, c1 - c0, M) for c0, c1 in self.ranges]            # each rank's dispatched part
        self.Z = [e(n_esp, E, c1 - c0, Hl) for c0, c1 in self.ranges]
        self.A = [e(n_esp, E, c1 - c0, Hl) for c0, c1 in self.ranges]
        self.Ypart = e(E, C, M)                                              # scratch for one rank's output
        self.Yret = e(n_esp, E, C, M); self.y = e(S, M)
        self.dw = e(S, k, dt=f32); self.dYpart = e(E, C, M); self.dXpart = e(E, C, M)
        self.dbuf = e(n_esp, E, C, M)
        self.dW1 = e(E, M, H); self.dW2 = e(E, H, M); self.dW1r = e(E, M, H); self.dW2r = e(E, H, M)
        self.dx = e(S, M); self.dlogits = e(S, E, dt=f32); self.dWg = e(M, E, dt=f32); self.dbias = e(E, dt=f32)
        cmax = max(c1 - c0 for c0, c1 in self.ranges)
        nbytes = max(api.moe_gate_workspace_bytes(S, E, k), api.moe_ffn_workspace_bytes(self.dt, 1, E, max(cmax, 1), M, H, n_esp),
                     api.moe_gate_bwd_workspace_bytes(S, M, E), 256)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def forward(self, x, Wg, bias, W1, W2):
        S, M, E, k, C, H = self.S, self.M, self.E, self.k, self.C, self.H
        self.x, self.Wg, self.W1, self.W2 = x, Wg, W1, W2
        api.moe_gate_topk(x, Wg, bias, S, M, E, k, C, 0, 1, self.norm_topk, self.logits, self.idx, self.slot, self.w,
                          self.inv, self.counts, self.ws)
        for r, (c0, c1) in enumerate(self.ranges):
            if c1 == c0:
                continue
            Cr = c1 - c0
            api.moe_dispatch_slots(x, S, M, E, k, C, c0, c1, self.inv, None, self.parts[r])
            for j in range(self.n_esp):
                Y = self.Ypart.view(-1)[:E * Cr * M].view(1, E, Cr, M)
                api.moe_expert_ffn_fwd(self.parts[r].view(1, E, Cr, M), W1, W2, 1, E, Cr, M, H, j, self.n_esp,
                                       self.Z[r][j], self.A[r][j], Y)
                self.Yret[j, :, c0:c1].copy_(Y[0])                           # MP-AllGather
        api.moe_combine_fwd(self.Yret, self.n_esp, S, M, E, k, C, self.idx, self.slot, self.w, self.y)
        return self.y

    def backward(self, dy):
        S, M, E, k, C, H = self.S, self.M, self.E, self.k, self.C, self.H
        api.moe_combine_bwd(dy, self.Yret, self.n_esp, S, M, E, k, C, self.idx, self.slot, self.inv, self.w, None, self.dw)
        self.dW1.zero_(); self.dW2.zero_(); self.dbuf.zero_()
        for r, (c0, c1) in enumerate(self.ranges):
            if c1 == c0:
                continue
            Cr = c1 - c0
            dYp = self.dYpart.view(-1)[:E * Cr * M].view(1, E, Cr, M)
            api.moe_dispatch_slots(dy, S, M, E, k, C, c0, c1, self.inv, self.w, dYp)
            for j in range(self.n_esp):
                dXp = self.dXpart.view(-1)[:E * Cr * M].view(1, E, Cr, M)
                api.moe_expert_ffn_bwd(dYp, self.parts[r].view(1, E, Cr, M), self.Z[r][j], self.A[r][j], self.W1, self.W2,
                                       1, E, Cr, M, H, j, self.n_esp, dXp, self.dW1r, self.dW2r, self.ws)
                self.dbuf[j, :, c0:c1].copy_(dXp[0])                         # MP-AllGather of the backward pass
                hs = slice(j * self.Hl, (j + 1) * self.Hl)
                self.dW1[:, :, hs] += self.dW1r[:, :, hs]                    # gradient reduction over the MP group
                self.dW2[:, hs, :] += self.dW2r[:, hs, :]
        api.moe_combine_fwd(self.dbuf, self.n_esp, S, M, E, k, C, self.idx, self.slot, None, self.dx)
        api.moe_gate_bwd(self.dw, self.w, self.idx, self.logits, self.x, self.Wg, S, M, E, k, self.norm_topk,
                         self.dlogits, self.dWg, self.dbias, self.dx, 1, self.ws)
        return self.dx
