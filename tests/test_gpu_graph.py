"""The whole step (top-k, routing sort, SMoE MLP forward and backward) recorded once into a HIP graph and
replayed: the library allocates nothing, never synchronises and records no memset, so a capture of the
caller's stream holds only its kernels.  Every replay is checked bit for bit against the same step run
eagerly on the same inputs, with eager work and synchronisations between the replays."""
import pytest
import torch

import smoe_inputs as si

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["C3-small", "C1"])
def test_step_replays_from_a_graph(name):
    import paper_2403_08245_amd as smoe
    cfg = si.CONFIGS[name]
    cases = [si.mlp_case(cfg, seed) for seed in (0, 1, 2)]
    dev = torch.device("cuda:0")
    names = ("logits", "X", "W1", "W2", "dY")
    static = {n: cases[0][n].to(dev).clone() for n in names}

    def step():
        ei, gates = smoe.topk_gate(static["logits"], cfg.k)
        r = smoe.route(ei, cfg.E)
        Y, buf = smoe.mlp_fwd(static["X"], static["W1"], static["W2"], r, cfg.k, gates, cfg.act)
        dX, dW1, dW2, dg = smoe.mlp_bwd(static["dY"], static["X"], static["W1"], static["W2"], r, cfg.k, gates, cfg.act, buf)
        return ei, gates, r.sorted_scattered_idxs, r.expert_offsets, Y, dX, dW1, dW2, dg

    side = torch.cuda.Stream()                      # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                   # warm-up outside the capture (one-time kernel attribute calls)
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        captured = step()
    for case in (cases[1], cases[2], cases[0], cases[1]):
        for n in names:
            static[n].copy_(case[n].to(dev))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in captured]
        eager = step()                              # eager work between the replays, same inputs
        torch.cuda.synchronize()
        for a, b in zip(got, eager):
            assert torch.equal(a, b)
