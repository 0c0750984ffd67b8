"""The library allocates nothing, clears nothing with memset calls and never synchronises: a whole step
(forward and backward) can be recorded into a HIP graph.  Every replay must reproduce the eager step bit
for bit, also with eager work and synchronisations between the replays."""
import pytest
import torch

from paper_2407_00599_amd import synth
from paper_2407_00599_amd.layer import MoERankLayer
from util import DEV, to_dev, torch_dtype

pytestmark = pytest.mark.gpu

NAMES = ("logits", "idx", "slot", "inv", "counts", "w", "y", "dx", "dW1", "dW2", "dWg", "dlogits")


@pytest.mark.parametrize("name,n_esp", [("tiny_fp32", 2), ("layer_bf16", 1)])
def test_step_replays_from_a_graph(name, n_esp):
    cfg = synth.CONFIGS[name]
    x = synth.tokens(cfg); Wg = synth.gate_weight(cfg); bias = synth.gate_bias(cfg)
    W1, W2 = synth.expert_weights(cfg, cfg.E); dy = to_dev(synth.upstream_grad(cfg))
    L = MoERankLayer(cfg.S_total, cfg.M, cfg.H, cfg.E, cfg.k, cfg.f, dtype=torch_dtype(cfg.dtype), n_mp=cfg.n_mp,
                     mp_idx=cfg.mp_idx, n_esp=n_esp, norm_topk=1, device=DEV)
    args = (to_dev(x), to_dev(Wg), to_dev(bias) if bias is not None else None, to_dev(W1), to_dev(W2))

    def step():
        L.forward(*args)
        L.backward(dy)

    step()
    torch.cuda.synchronize()
    ref = {n: getattr(L, n).clone() for n in NAMES}
    side = torch.cuda.Stream()                      # warm-up on a side stream, as graph capture requires
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        for n in NAMES:
            getattr(L, n).fill_(-3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in NAMES:
            assert torch.equal(getattr(L, n), ref[n]), n
        step()                                      # eager work between the replays
        torch.cuda.synchronize()
