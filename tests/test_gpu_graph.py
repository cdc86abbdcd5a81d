"""The hot path under HIP-graph capture: the library enqueues kernels only (no allocation, no memset, no
synchronisation), so a training step captured once must replay with the results of the eager step, on every replay,
with other work and synchronisations between the replays."""
import pytest
import torch

import paper_2407_11062_amd as eq
from paper_2407_11062_amd import synth

pytestmark = pytest.mark.gpu


def test_block_ap_and_e2e_steps_replay_from_a_graph():
    T, I, O, bits, g = 300, 384, 264, 2, 64
    dev = torch.device("cuda:0")
    W = synth.normal((O, I), 0.02, synth.seed_of("graph", "W"), torch.bfloat16).to(dev)
    s, z = eq.eqat_init_minmax(W, bits, g)
    Wp, zp = eq.eqat_pack(W, s, z, bits, g)
    X = torch.empty((T, I), dtype=torch.bfloat16, device=dev)
    Yref = torch.empty((T, O), dtype=torch.bfloat16, device=dev)
    d = eq.make_desc(T, I, O, bits, g, eq.BF16, eq.BF16)

    def buffers():
        return {"Y": torch.empty((T, O), dtype=torch.bfloat16, device=dev), "loss": torch.empty(1, device=dev),
                "dY": torch.empty((T, O), dtype=torch.bfloat16, device=dev),
                "out": {"dX": torch.empty((T, I), dtype=torch.bfloat16, device=dev), "dW": torch.empty_like(W),
                        "ds": torch.empty_like(s), "dz": torch.empty_like(s)},
                "Yq": torch.empty((T, O), dtype=torch.bfloat16, device=dev),
                "outq": {"dX": torch.empty((T, I), dtype=torch.bfloat16, device=dev), "ds": torch.empty_like(s)},
                "ws": eq.workspace(d, eq.OP_FQ_BWD, dev), "wsq": eq.workspace(d, eq.OP_Q_BWD, dev),
                "lws": torch.empty(eq.lib().eqat_recon_loss_workspace_bytes(), dtype=torch.uint8, device=dev)}

    def step(b):
        eq.eqat_fq_linear_fwd(X, W, s, z, bits, g, Y=b["Y"], ws=b["ws"], keep=True)
        eq.eqat_recon_loss(b["Y"], Yref, loss=b["loss"], dY=b["dY"], ws=b["lws"])
        eq.eqat_fq_linear_bwd(X, W, s, z, b["dY"], bits, g, out=b["out"], ws=b["ws"], kept=True)
        eq.eqat_qlinear_fwd(X, Wp, s, zp, bits, g, Y=b["Yq"], ws=b["wsq"], keep=True)
        eq.eqat_qlinear_bwd(X, Wp, s, zp, b["dY"], I, bits, g, out=b["outq"], ws=b["wsq"], kept=True)

    def new_inputs(k):
        X.copy_(synth.normal((T, I), 1.0, synth.seed_of("graph", "X", k), torch.bfloat16))
        Yref.copy_(synth.normal((T, O), 0.3, synth.seed_of("graph", "Yref", k), torch.bfloat16))

    eager, graphed = buffers(), buffers()
    new_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graphed)                                   # first use outside the capture (one-time kernel attributes)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(graphed)
    for k in range(1, 5):
        new_inputs(k)
        step(eager)
        scratch = torch.randn(1 << 20, device=dev).sum()        # the program's own eager work between replays
        torch.cuda.synchronize()
        for t in (graphed["Y"], graphed["dY"], graphed["Yq"], *graphed["out"].values(), *graphed["outq"].values()):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(scratch)
        assert torch.equal(graphed["Y"], eager["Y"]) and torch.equal(graphed["loss"], eager["loss"]), k
        assert torch.equal(graphed["Yq"], eager["Yq"]), k
        for name in ("dX", "dW", "ds", "dz"):
            assert torch.equal(graphed["out"][name], eager["out"][name]), (k, name)
        for name in ("dX", "ds"):
            assert torch.equal(graphed["outq"][name], eager["outq"][name]), (k, name)
