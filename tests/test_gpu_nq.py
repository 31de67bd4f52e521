"""GPU parity of the unquantised variant (LoQT-nq: W and P in bf16): loqt_linear_fwd_nq / loqt_linear_bwd_nq /
loqt_merge_nq against the oracle."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth

pytestmark = pytest.mark.gpu
TOL = 2e-2


@pytest.fixture(params=["auto", "factored", "folded"], autouse=True)
def path(request):
    """Every test runs under each form of the rank-r term: carried as a second K segment, folded into a
    transient copy of the weight, or chosen by the token count."""
    from paper_2405_16528_amd import binding as L
    L.set_path({"auto": L.PATH_AUTO, "factored": L.PATH_PREPASS, "folded": L.PATH_FOLDED}[request.param])
    yield request.param
    L.set_path(L.PATH_AUTO)


def _setup(T, out, inp, r, seed, sigma_B=2e-2):
    from tests import gpu_util as G
    rng = synth.rng_for(seed, "nq-gpu", str(T), str(out), str(inp), str(r))
    W = synth.normal_bf16(rng, (out, inp), 0.02)
    P = O.f32_to_bf16_rne(synth.orthonormal_f32(rng, out, r))
    B = synth.normal_bf16(rng, (r, inp), sigma_B)
    x = synth.normal_bf16(rng, (T, inp), 1.0)
    dy = synth.normal_bf16(rng, (T, out), 1e-2)
    dev = {k: G.bf16_dev(v) for k, v in dict(W=W, P=P, B=B, x=x, dy=dy).items()}
    return W, P, B, x, dy, dev


@pytest.mark.parametrize("T,out,inp,r", [(256, 512, 512, 128), (300, 520, 456, 128), (130, 300, 1000, 64),
                                         (515, 1100, 333, 192), (1300, 768, 1365, 256)])
@pytest.mark.parametrize("s", [1.0, 0.25])
def test_fwd_bwd_parity(T, out, inp, r, s):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    W, P, B, x, dy, d = _setup(T, out, inp, r, seed=T + out)
    y = G.bf16_empty(T, out, fill=float("nan"))
    L.loqt_linear_fwd_nq(d["x"], d["W"], d["P"], d["B"], s, y, G.workspace(L.OP_FWD_NQ, T, out, inp, r))
    dx = G.bf16_empty(T, inp, fill=float("nan"))
    dB = torch.full((r, inp), float("nan"), dtype=torch.float32, device="cuda")
    L.loqt_linear_bwd_nq(d["dy"], d["x"], d["W"], d["P"], d["B"], s, dx, dB, False,
                         G.workspace(L.OP_BWD_NQ, T, out, inp, r))
    torch.cuda.synchronize()
    y_ref = O.loqt_linear_fwd_nq(x, W, P, B, s)
    dx_ref, dB_ref = O.loqt_linear_bwd_nq(dy, x, W, P, B, s)
    ey = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(y)), y_ref)
    ex = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dx)), dx_ref)
    eb = G.max_err_over_rms(dB.cpu().numpy().astype(np.float64), dB_ref)
    print(f"nq T={T} out={out} in={inp} r={r} s={s}: err/rms y {ey:.2e} dx {ex:.2e} dB {eb:.2e}")
    assert ey <= TOL and ex <= TOL and eb <= TOL


def test_bwd_options():
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    T, out, inp, r = 300, 260, 200, 64
    W, P, B, x, dy, d = _setup(T, out, inp, r, seed=9)
    ws = G.workspace(L.OP_BWD_NQ, T, out, inp, r)
    _, dB_ref = O.loqt_linear_bwd_nq(dy, x, W, P, B, 0.5)
    base = synth.normal_f32(synth.rng_for(9, "nq-base"), (r, inp), float(np.sqrt(np.mean(dB_ref ** 2))))
    dB = torch.from_numpy(base.copy()).cuda()
    L.loqt_linear_bwd_nq(d["dy"], d["x"], d["W"], d["P"], d["B"], 0.5, None, dB, True, ws)
    dB16 = G.bf16_empty(r, inp, fill=float("nan"))
    L.loqt_linear_bwd_nq(d["dy"], d["x"], d["W"], d["P"], d["B"], 0.5, None, dB16, False, ws)
    torch.cuda.synchronize()
    assert G.max_err_over_rms(dB.cpu().numpy().astype(np.float64), base + dB_ref) <= TOL
    assert G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dB16)), dB_ref) <= TOL


@pytest.mark.parametrize("out,inp,r", [(512, 512, 128), (300, 456, 64), (1100, 333, 192), (260, 2048, 256)])
def test_merge(out, inp, r):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    W, P, B, x, dy, d = _setup(8, out, inp, r, seed=out + inp, sigma_B=5e-3)
    # B = 0: W comes back bit for bit (and the pitch padding is not touched)
    Wz = G.bf16_dev(W)
    L.loqt_merge_nq(Wz, d["P"], G.bf16_dev(np.zeros_like(B)), 1.0)
    torch.cuda.synchronize()
    assert np.array_equal(G.bf16_host(Wz), W)
    for s in (1.0, 0.25):
        Wm = G.bf16_dev(W)
        L.loqt_merge_nq(Wm, d["P"], d["B"], s)
        torch.cuda.synchronize()
        got = G.bf16_host(Wm)
        exact = O.loqt_merge_nq_f64(W, P, B, s)
        # the stored bf16 is the rounding of the device's fp32 sum, which differs from the exact sum by the
        # fp32 roundings of the product and the addition (absolute, so it matters where W + s P B cancels)
        err = np.abs(O.bf16_to_f64(got) - exact)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact), 1e-30))) - 7)
        fp32_err = (np.abs(O.bf16_to_f64(W)) + abs(s) * (np.abs(O.bf16_to_f64(P)) @ np.abs(O.bf16_to_f64(B)))) * 2.0 ** -21
        assert np.all(err <= 0.5 * ulp + fp32_err), float(((err - fp32_err) / ulp).max())
        ref = O.loqt_merge_nq(W, P, B, s)
        rate = float(np.mean(got != ref))
        print(f"nq merge {out}x{inp} r={r} s={s}: bf16 results differing from the oracle's rounding {rate:.2e}")
        assert rate <= 2e-3
