"""Pins for the oracle's LoQT-nq functions (the layer with W and P in 16 bits): loops, the projected
full gradient, exact finite differences, and agreement with the quantised layer's functions on weights
that both can represent exactly."""
import numpy as np
import pytest

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth


def _tiny(seed=0, T=4, out=66, inp=70, r=64):
    rng = synth.rng_for(seed, "nq", str(out), str(inp))
    W = synth.normal_bf16(rng, (out, inp), 0.02)
    P = O.f32_to_bf16_rne(synth.orthonormal_f32(rng, out, r))
    B = synth.normal_bf16(rng, (r, inp), 0.05)
    x = synth.normal_bf16(rng, (T, inp), 1.0)
    dy = synth.normal_bf16(rng, (T, out), 1e-2)
    return W, P, B, x, dy


def test_against_loops_and_projected_gradient():
    W, P, B, x, dy = _tiny()
    s = 0.5
    Wd, Pd, Bd, xd, dyd = (O.bf16_to_f64(a) for a in (W, P, B, x, dy))
    out, inp = Wd.shape
    r = Pd.shape[1]
    Weff = np.zeros((out, inp))
    for o in range(out):
        for i in range(inp):
            Weff[o, i] = Wd[o, i] + s * sum(Pd[o, k] * Bd[k, i] for k in range(r))
    assert np.allclose(O.loqt_merge_nq_f64(W, P, B, s), Weff, rtol=1e-12, atol=1e-16)
    assert np.allclose(O.loqt_linear_fwd_nq(x, W, P, B, s), xd @ Weff.T, rtol=1e-10, atol=1e-14)
    dx, dB = O.loqt_linear_bwd_nq(dy, x, W, P, B, s)
    assert np.allclose(dx, dyd @ Weff, rtol=1e-10, atol=1e-16)
    assert np.allclose(dB, s * Pd.T @ (dyd.T @ xd), rtol=1e-10, atol=1e-16)   # G^B = P^T G^W (sec. 2.2)
    E = np.random.default_rng(0).standard_normal(Bd.shape)
    y_shift = xd @ (Wd + s * Pd @ (Bd + E)).T
    assert np.sum(dyd * (y_shift - xd @ Weff.T)) == pytest.approx(np.sum(dB * E), rel=1e-9)


def test_agrees_with_the_quantised_layer_on_exactly_representable_weights():
    """Codes in {0, 7, 15} (levels -1, 0, 1) with power-of-two absmax dequantise to values bf16 holds exactly."""
    rng = np.random.default_rng(1)
    out, inp, r, T = 64, 128, 64, 5
    wc = rng.choice(np.array([0, 7, 15], dtype=np.uint8), (out, inp)); wc[:, ::64] = 15
    wa = np.full((out, inp // 64), 2.0 ** -5, dtype=np.float32)
    pc = rng.choice(np.array([0, 7, 15], dtype=np.uint8), (out, r)); pc[:, 0] = 15
    pa = np.full((out, 1), 2.0 ** -3, dtype=np.float32)
    W = O.f32_to_bf16_rne(O.nf4_dequantize_f32(wc, wa))
    P = O.f32_to_bf16_rne(O.nf4_dequantize_f32(pc, pa))
    assert np.array_equal(O.bf16_to_f64(W), O.nf4_dequantize_f64(wc, wa))
    g = synth.rng_for(1, "nq-rep")
    B, x, dy = synth.normal_bf16(g, (r, inp), 0.01), synth.normal_bf16(g, (T, inp), 1.0), synth.normal_bf16(g, (T, out), 0.01)
    assert np.array_equal(O.loqt_linear_fwd_nq(x, W, P, B, 0.25), O.loqt_linear_fwd(x, (wc, wa), (pc, pa), B, 0.25))
    a, b = O.loqt_linear_bwd_nq(dy, x, W, P, B, 0.25), O.loqt_linear_bwd(dy, x, (wc, wa), (pc, pa), B, 0.25)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(O.loqt_merge_nq_f64(W, P, B, 0.25), O.loqt_merge_f64((wc, wa), (pc, pa), B, 0.25))


def test_merge_rounding_and_noop():
    W, P, B, x, dy = _tiny(seed=2)
    assert np.array_equal(O.loqt_merge_nq(W, P, np.zeros_like(B), 1.0), W)
    m = O.loqt_merge_nq(W, P, B, 1.0)
    exact = O.loqt_merge_nq_f64(W, P, B, 1.0)
    assert np.all(np.abs(O.bf16_to_f64(m) - exact) <= np.abs(exact) * 2.0 ** -8 + 1e-30)  # half a bf16 ulp
