"""The hot path under HIP graph capture: a captured forward + backward + merge must replay with the same
results as the eager calls, on every replay (the library allocates nothing, records no memset nodes and
keeps no state between calls; one eager warm-up call per kernel configures its LDS size before capture)."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_eager():
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    T, out, inp, r, s = 1100, 640, 520, 128, 0.5
    lay = synth.make_layer("graph", "l", out, inp, r, T, 5)
    Wq, Pq = O.nf4_quantize(lay.W), O.nf4_quantize(lay.P)
    d = dict(x=G.bf16_dev(lay.x), dy=G.bf16_dev(lay.dy), B=G.bf16_dev(lay.B), Wq=G.nf4_dev(*Wq), Pq=G.nf4_dev(*Pq))
    ws = torch.empty(max(L.loqt_workspace_bytes(op, T, out, inp, r) for op in (L.OP_FWD, L.OP_BWD, L.OP_MERGE)),
                     dtype=torch.uint8, device="cuda")
    y, dx = G.bf16_empty(T, out), G.bf16_empty(T, inp)
    dB = torch.empty((r, inp), dtype=torch.float32, device="cuda")
    merged = L.NF4Tensor.empty(out, inp)

    def step():
        L.loqt_linear_fwd(d["x"], d["Wq"], d["Pq"], d["B"], s, y, ws)
        L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], s, dx, dB, False, ws)
        L.loqt_merge_requant(d["Wq"], d["Pq"], d["B"], s, out=merged, ws=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # eager warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = [t.clone() for t in (y, dx, dB, merged.codes, merged.absmax)]

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(3):
        for t in (y, dx, dB, merged.codes, merged.absmax):
            t.zero_() if t.dtype != torch.bfloat16 else t.fill_(0)
        # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((y, dx, dB, merged.codes, merged.absmax), eager):
            assert torch.equal(got, ref), f"replay {rep} differs from the eager result"


_COLD_CAPTURE = r"""
import sys
import numpy as np, torch
sys.path.insert(0, {root!r})
from paper_2405_16528_amd import binding as L
torch.cuda.set_device(0)
L.loqt_prepare()                       # instead of an eager warm-up of every kernel configuration
g = torch.Generator(device="cuda"); g.manual_seed(3)
T, out, inp, r, s = 1100, 1280, 1024, 128, 0.5     # in >= 1024: the merge takes the grouped pre-pass form
rb = lambda a, b, sig: (torch.randn((a, b), device="cuda", generator=g) * sig).to(torch.bfloat16)
Wq = L.nf4_quantize(torch.randn((out, inp), device="cuda", generator=g) * 0.02)
Pq = L.nf4_quantize(torch.randn((out, r), device="cuda", generator=g) / out ** 0.5)
B, x, dy = rb(r, inp, 2e-2), rb(T, inp, 1.0), rb(T, out, 1e-2)
ws = torch.empty(max(L.loqt_workspace_bytes(op, T, out, inp, r) for op in (L.OP_FWD, L.OP_BWD, L.OP_MERGE)),
                 dtype=torch.uint8, device="cuda")
y = torch.zeros((T, out), dtype=torch.bfloat16, device="cuda"); dx = torch.zeros((T, inp), dtype=torch.bfloat16, device="cuda")
dB = torch.zeros((r, inp), dtype=torch.float32, device="cuda"); merged = L.NF4Tensor.empty(out, inp)
scales = Wq.absmax.reshape(-1)
codes8 = torch.zeros(scales.numel(), dtype=torch.uint8, device="cuda")
c1 = torch.zeros((scales.numel() + 255) // 256, dtype=torch.float32, device="cuda"); mean = torch.zeros(1, device="cuda")
descs = L.make_merge_descs([(Wq, merged, Pq, B, s)])
def step():
    L.loqt_linear_fwd(x, Wq, Pq, B, s, y, ws)
    L.loqt_linear_bwd(dy, x, Wq, Pq, B, s, dx, dB, False, ws)
    L.loqt_merge_requant_batched(descs, ws)
    L.loqt_absmax_dq_compress_static(scales, codes8, c1, mean)
outs = (y, dx, dB, merged.codes, merged.absmax, codes8, c1, mean)
side = torch.cuda.Stream()
side.wait_stream(torch.cuda.current_stream())
graph = torch.cuda.CUDAGraph()
with torch.cuda.graph(graph, stream=side):    # the very first launches of this process are recorded, not run
    step()
graph.replay(); torch.cuda.synchronize()
first = [t.clone() for t in outs]
for t in outs:
    t.zero_()
step(); torch.cuda.synchronize()              # eager, afterwards
assert all(torch.equal(a, b) for a, b in zip(first, outs)), "captured first call differs from the eager one"
assert float(y.float().abs().max()) > 0 and float(dB.abs().max()) > 0
for t in outs:
    t.zero_()
graph.replay(); torch.cuda.synchronize()
assert all(torch.equal(a, b) for a, b in zip(first, outs)), "second replay differs"
print("cold capture ok")
"""


def test_first_call_can_be_captured_after_prepare():
    """A fresh process: loqt_prepare(), then the first forward + backward + merge + static scale compression of the
    process are recorded into a graph without any eager warm-up, replayed, and compared with eager calls."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", _COLD_CAPTURE.format(root=root)], capture_output=True, text=True,
                         timeout=240)
    assert res.returncode == 0 and "cold capture ok" in res.stdout, res.stdout[-2000:] + res.stderr[-4000:]
