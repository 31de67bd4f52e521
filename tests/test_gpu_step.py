"""GPU parity of loqt_adam_step (Alg. 1 line 9) and loqt_merge_dense (Alg. 1 line 5) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rows,cols,gdtype", [(128, 512, "f32"), (77, 333, "f32"), (64, 1000, "bf16")])
def test_adam_steps(rows, cols, gdtype):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    rng = synth.rng_for(3, "adam", str(rows), str(cols))
    Bb = synth.normal_bf16(rng, (rows, cols), 1e-2)
    Bd = G.bf16_dev(Bb)
    m = torch.zeros((rows, cols), dtype=torch.float32, device="cuda")
    v = torch.zeros_like(m)
    Bo, mo, vo = O.bf16_to_f64(Bb), np.zeros((rows, cols)), np.zeros((rows, cols))
    # the C ABI takes the hyper-parameters as floats: give the oracle the same (rounded) values
    lr, b1, b2, eps = (float(np.float32(h)) for h in (1e-3, 0.9, 0.95, 1e-8))
    for t in range(1, 6):
        g32 = synth.normal_f32(rng, (rows, cols), 3e-4 * t)
        if gdtype == "bf16":
            gb = O.f32_to_bf16_rne(g32)
            gd, g64 = G.bf16_dev(gb), O.bf16_to_f64(gb)
        else:
            gd, g64 = torch.from_numpy(g32).cuda(), g32.astype(np.float64)
        L.loqt_adam_step(Bd, gd, m, v, lr, t, beta1=b1, beta2=b2, eps=eps)
        torch.cuda.synchronize()
        Bn, mo, vo = O.adam_step(Bo, g64, mo, vo, lr, b1, b2, eps, t)
        got = G.bf16_host(Bd)
        ref = O.f32_to_bf16_rne(Bn.astype(np.float32))
        # fp32 arithmetic on the device against fp64: the bf16 result may land on the neighbouring value
        # when the exact result sits next to a rounding boundary
        d = np.abs(got.astype(np.int32) - ref.astype(np.int32))
        assert d.max() <= 1 and np.mean(d != 0) <= 2e-3, (d.max(), np.mean(d != 0))
        # fp32 moments against fp64: a few ulp, measured against the largest entry (sums can cancel)
        assert np.abs(m.cpu().numpy() - mo).max() <= 1e-6 * np.abs(mo).max()
        assert np.abs(v.cpu().numpy() - vo).max() <= 1e-6 * np.abs(vo).max()
        Bo = O.bf16_to_f64(got)  # continue from the device's B so one rounding flip does not compound


@pytest.mark.parametrize("out,inp,r,s", [(512, 512, 128, 1.0), (300, 456, 64, 0.25), (1100, 333, 192, 0.5)])
def test_merge_dense(out, inp, r, s):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    lay = synth.make_layer("dense", "l", out, inp, r, 8, out + inp)
    lay.B = synth.normal_bf16(synth.rng_for(out, "dense-B"), (r, inp), 2e-2)
    Wq, Pq = O.nf4_quantize(lay.W), O.nf4_quantize(lay.P)
    dWq, dPq, dB = G.nf4_dev(*Wq), G.nf4_dev(*Pq), G.bf16_dev(lay.B)
    ld = (inp + 3) // 4 * 4
    Wd = torch.full((out, ld), float("nan"), dtype=torch.float32, device="cuda")[:, :inp]
    L.loqt_merge_dense(dWq, dPq, dB, s, Wd)
    torch.cuda.synchronize()
    got = Wd.cpu().numpy().astype(np.float64)
    ref = O.loqt_merge_dense_f32(Wq, Pq, lay.B, s).astype(np.float64)
    old = O.nf4_dequantize_f64(*Wq)
    # the error lives in the rank-r product (bf16 operands): measure it against that term
    upd_err = np.abs((got - old) - (ref - old)).max() / np.sqrt(np.mean((ref - old) ** 2))
    print(f"merge_dense {out}x{inp} r={r}: update err/rms {upd_err:.2e}")
    assert upd_err <= 2e-2
    # quantising the dense result on the device is the fused merge, bit for bit
    q1 = L.nf4_quantize(Wd)
    q2 = L.loqt_merge_requant(dWq, dPq, dB, s, out=L.NF4Tensor.empty(out, inp))
    torch.cuda.synchronize()
    c1, a1, _, _ = G.nf4_host(q1)
    c2, a2, _, _ = G.nf4_host(q2)
    assert np.array_equal(c1, c2) and np.array_equal(a1, a2)
    # B = 0: the dense merge is the fp32 dequantisation
    Z = G.bf16_dev(np.zeros_like(lay.B))
    L.loqt_merge_dense(dWq, dPq, Z, s, Wd)
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy(), O.nf4_dequantize_f32(*Wq))
