"""The layer step under HIP graph capture: the library allocates nothing and never synchronises,
so a forward+backward step can be captured once and replayed; every replay must reproduce the
eager result bit for bit (with eager work and synchronisations between the replays)."""
import pytest
import torch

import mtf_inputs
from helpers import on_device, WEIGHT_DIMS

pytestmark = pytest.mark.gpu


def test_layer_step_replays_identically_from_a_graph():
    import paper_1811_02084_amd as mtf
    cfg = mtf_inputs.layer_inputs(27, 2, 192, 256, 2, 128, 512, 64, 16384)
    g = on_device(cfg)
    w = {k: g[k] for k in WEIGHT_DIMS}
    bufs = mtf.layer_alloc(g["x"], w)

    def step():
        mtf.layer_fwd(g["x"], w, cfg["scale"], True, bufs)
        mtf.layer_bwd(g["x"], w, bufs["saved"], g["dz"], cfg["scale"], True, bufs)

    step()
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in bufs["grads"].items()}
    eager.update(z=bufs["z"].clone(), dx=bufs["dx"].clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        for t in list(bufs["grads"].values()) + [bufs["z"], bufs["dx"]]:
            t.fill_(float("nan"))                # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in bufs["grads"].items():
            assert torch.equal(v, eager[k]), (replay, k)
        assert torch.equal(bufs["z"], eager["z"]) and torch.equal(bufs["dx"], eager["dx"]), replay
