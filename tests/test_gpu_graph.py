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
