"""The layer step under HIP graph capture.

Every C-ABI call only enqueues kernels on the caller's stream (no allocation, no memset node, no host
synchronisation), so a whole forward + backward step can be captured once and replayed.  The test replays the
graph several times, with eager work of the program and synchronisations between the replays, and checks every
replay against the eager result bit for bit - for the plain pair of FFN calls and for the pair that saves products."""
import pytest
import torch

from paper_2602_11686_amd import inputs as I
from paper_2602_11686_amd.layer import MoeLayerBuffers
from gpu_common import dev, shape_of

pytestmark = pytest.mark.gpu

BASE = I.WORKLOADS["cfg2_e64k4"]


@pytest.mark.parametrize("products", [False, True])
def test_a_captured_step_replays_bit_for_bit(products):
    w = I.scaled(BASE, name="graph", seed=31, T=1536, d=512, f=640, E=24, k=4, dtype="bf16", zipf_s=1.0, backward=True,
                 target_ratio=None, alpha=0.8, dead=2)
    inp = I.layer_inputs(w)
    g = {n: dev(v, w) if n != "bias" else torch.from_numpy(v).cuda() for n, v in inp.items()}
    s = shape_of(w)
    buf = MoeLayerBuffers(s, backward=True, save_products=products)
    outs = lambda: (buf.y, buf.dx, buf.dw1, buf.dw3, buf.dw2, buf.dw_gate, buf.topk_ids, buf.row_of_pair)

    def step():
        buf.forward(g["x"], g["w_gate"], g["bias"], g["w1"], g["w3"], g["w2"])
        buf.backward(g["x"], g["w_gate"], g["w1"], g["w3"], g["w2"], g["dy"])

    step()                       # eager: also sets the one-time kernel attributes and the device check
    torch.cuda.synchronize()
    want = [t.clone() for t in outs()]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                   # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        for t in outs():         # eager work between the replays: every output is wiped
            if t.dtype.is_floating_point:
                t.fill_(float("nan"))
            else:
                t.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("y", "dx", "dw1", "dw3", "dw2", "dw_gate", "ids", "row_of_pair"), outs(), want):
            assert torch.equal(a, b), (name, "replay", rep)
