"""Pins for the oracle's forward / backward / merge (paper sec. 2.2, 2.4, Alg. 1):
brute-force loops, the other association of the products, library routines on the
special cases that reduce to them, and exact finite differences."""
import numpy as np
import pytest

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth


def _tiny(seed=0, T=5, out=70, inp=130, r=64):
    L = synth.make_layer("tiny", "l", out, inp, r, T, seed)
    Wq = O.nf4_quantize(L.W)
    Pq = O.nf4_quantize(L.P)
    # make B large enough that the low-rank term is far from negligible
    B = synth.normal_bf16(synth.rng_for(seed, "tinyB"), (r, inp), 0.05)
    return L, Wq, Pq, B


def _loops_weff(Wq, Pq, B, s):
    """W_eff[o,i] = M*q[code] + s * sum_k P[o,k] B[k,i], written out element by element."""
    codes, am = Wq
    pc, pam = Pq
    Bd = O.bf16_to_f64(B)
    out, inp = codes.shape
    r = pc.shape[1]
    W = np.zeros((out, inp))
    for o in range(out):
        for i in range(inp):
            acc = float(am[o, i // 64]) * float(O.NF4_LEVELS[codes[o, i]])
            lr = 0.0
            for k in range(r):
                lr += float(pam[o, k // 64]) * float(O.NF4_LEVELS[pc[o, k]]) * Bd[k, i]
            W[o, i] = acc + s * lr
    return W


@pytest.mark.parametrize("s", [1.0, 0.5, 0.25])
def test_fwd_bwd_against_loops(s):
    L, Wq, Pq, B = _tiny(T=3, out=66, inp=70, r=64)
    Weff = _loops_weff(Wq, Pq, B, s)
    xd, dyd = O.bf16_to_f64(L.x), O.bf16_to_f64(L.dy)
    y = O.loqt_linear_fwd(L.x, Wq, Pq, B, s)
    T, out, inp = 3, 66, 70
    y_ref = np.zeros((T, out))
    for t in range(T):
        for o in range(out):
            y_ref[t, o] = sum(xd[t, i] * Weff[o, i] for i in range(inp))
    assert np.allclose(y, y_ref, rtol=1e-12, atol=1e-14)
    dx, dB = O.loqt_linear_bwd(L.dy, L.x, Wq, Pq, B, s)
    dx_ref = np.zeros((T, inp))
    for t in range(T):
        for i in range(inp):
            dx_ref[t, i] = sum(dyd[t, o] * Weff[o, i] for o in range(out))
    assert np.allclose(dx, dx_ref, rtol=1e-12, atol=1e-16)
    # merge: same W_eff, then the codec (pinned separately)
    assert np.allclose(O.loqt_merge_f64(Wq, Pq, B, s), Weff, rtol=1e-12, atol=1e-16)


def test_fwd_reduces_to_library_matmul_when_B_is_zero():
    L, Wq, Pq, B = _tiny()
    B0 = np.zeros_like(B)
    y = O.loqt_linear_fwd(L.x, Wq, Pq, B0, 0.5)
    Wd = O.nf4_dequantize_f32(*Wq).astype(np.float64)  # fp32-rounded weights: compare loosely
    assert np.allclose(y, O.bf16_to_f64(L.x) @ Wd.T, rtol=1e-6, atol=1e-7)
    dx, dB = O.loqt_linear_bwd(L.dy, L.x, Wq, Pq, B0, 0.5)
    assert np.allclose(dx, O.bf16_to_f64(L.dy) @ Wd, rtol=1e-6, atol=1e-9)


def test_merge_keeps_the_function():
    # sec. 2: W_T = W_{T-1} + P B  => forward through (W_q, P_q, B) equals forward through
    # the merged, not yet requantised, weight
    L, Wq, Pq, B = _tiny(seed=2)
    for s in (1.0, 0.25):
        y = O.loqt_linear_fwd(L.x, Wq, Pq, B, s)
        Wm = O.loqt_merge_f64(Wq, Pq, B, s)
        assert np.allclose(y, O.bf16_to_f64(L.x) @ Wm.T, rtol=1e-11, atol=1e-13)
        dx, _ = O.loqt_linear_bwd(L.dy, L.x, Wq, Pq, B, s)
        assert np.allclose(dx, O.bf16_to_f64(L.dy) @ Wm, rtol=1e-11, atol=1e-15)


def test_dB_is_projected_full_gradient():
    # sec. 2.2: G^B = P^T G^W with G^W = dy^T x (full out x in, only formed here)
    L, Wq, Pq, B = _tiny(seed=3, T=9, out=96, inp=70, r=64)
    s = 0.5
    _, dB = O.loqt_linear_bwd(L.dy, L.x, Wq, Pq, B, s)
    GW = O.bf16_to_f64(L.dy).T @ O.bf16_to_f64(L.x)
    Pd = O.nf4_dequantize_f64(*Pq)
    ref = s * (Pd.T @ GW)
    assert dB.shape == (64, 70)
    assert np.abs(dB - ref).max() <= 1e-12 * np.sqrt(np.mean(ref ** 2))


def test_dB_and_dx_by_exact_finite_differences():
    # L = <y, dy> is linear in B and in x, so differences are exact up to rounding
    L, Wq, Pq, B = _tiny(seed=4, T=6, out=72, inp=130, r=64)
    s = 0.25
    dyd = O.bf16_to_f64(L.dy)
    dx, dB = O.loqt_linear_bwd(L.dy, L.x, Wq, Pq, B, s)
    rng = np.random.default_rng(0)
    y0 = O.loqt_linear_fwd(L.x, Wq, Pq, B, s)
    # perturb single entries of B by one bf16-representable step
    for _ in range(20):
        k, i = rng.integers(0, 64), rng.integers(0, 130)
        B1 = B.copy()
        B1[k, i] = B1[k, i] ^ 0x0040  # flip a mantissa bit: stays a finite bf16
        eps = O.bf16_to_f64(B1[k:k + 1, i:i + 1])[0, 0] - O.bf16_to_f64(B[k:k + 1, i:i + 1])[0, 0]
        y1 = O.loqt_linear_fwd(L.x, Wq, Pq, B1, s)
        lhs = np.sum((y1 - y0) * dyd)
        assert abs(lhs - eps * dB[k, i]) <= 1e-9 * abs(eps * dB[k, i]) + 1e-22
    for _ in range(20):
        t, i = rng.integers(0, 6), rng.integers(0, 130)
        x1 = L.x.copy()
        x1[t, i] = x1[t, i] ^ 0x0040
        eps = O.bf16_to_f64(x1[t:t + 1, i:i + 1])[0, 0] - O.bf16_to_f64(L.x[t:t + 1, i:i + 1])[0, 0]
        y1 = O.loqt_linear_fwd(x1, Wq, Pq, B, s)
        lhs = np.sum((y1 - y0) * dyd)
        assert abs(lhs - eps * dx[t, i]) <= 1e-9 * abs(eps * dx[t, i]) + 1e-22


def test_shapes_are_not_transposed():
    # non-square everything: a transposed operand cannot even multiply
    L, Wq, Pq, B = _tiny(seed=5, T=7, out=133, inp=150, r=128)
    y = O.loqt_linear_fwd(L.x, Wq, Pq, B, 1.0)
    dx, dB = O.loqt_linear_bwd(L.dy, L.x, Wq, Pq, B, 1.0)
    assert y.shape == (7, 133) and dx.shape == (7, 150) and dB.shape == (128, 150)
    c, a = O.loqt_merge_requant(Wq, Pq, B, 1.0)
    assert c.shape == (133, 150) and a.shape == (133, 3)


def test_merge_with_zero_B_is_a_noop():
    L, Wq, Pq, B = _tiny(seed=6, out=64, inp=256)
    c, a = O.loqt_merge_requant(Wq, Pq, np.zeros_like(B), 0.5)
    assert np.array_equal(c, Wq[0]) and np.array_equal(a, Wq[1])


def test_merge_exact_case():
    # W codes in {0, 7, 15} (values -M, 0, +M) with absmax M = 2^k; P codes in {0, 7, 15}
    # with absmax 2^-5; B small integers * 2^-10; s = 0.5: every product and sum is exact,
    # so the merged weight is known in closed form and so are its codes.
    rng = np.random.default_rng(7)
    out, inp, r = 8, 128, 64
    wc = rng.choice(np.array([0, 7, 15], dtype=np.uint8), (out, inp))
    wc[:, 0] = 15
    wc[:, 64] = 0
    wam = np.float32(2.0) ** rng.integers(-12, -9, (out, 2)).astype(np.float32)
    pc = rng.choice(np.array([0, 7, 15], dtype=np.uint8), (out, r))
    pc[:, 0] = 15
    pam = np.full((out, 1), 2.0 ** -5, dtype=np.float32)
    Bf = (rng.integers(-4, 5, (r, inp)) * 2.0 ** -10).astype(np.float32)
    B = synth.to_bf16_bits(Bf)
    assert np.array_equal(O.bf16_to_f64(B), Bf.astype(np.float64))
    s = 0.5
    Pv = np.where(pc == 15, 1.0, np.where(pc == 0, -1.0, 0.0)) * 2.0 ** -5
    Wv = O.NF4_LEVELS[wc] * np.repeat(wam.astype(np.float64), 64, axis=1)
    Wnew = Wv + s * (Pv @ Bf.astype(np.float64))
    assert np.array_equal(Wnew.astype(np.float32).astype(np.float64), Wnew)  # exact in fp32
    got = O.loqt_merge_f64((wc, wam), (pc, pam), B, s)
    assert np.array_equal(got, Wnew)
    c, a = O.loqt_merge_requant((wc, wam), (pc, pam), B, s)
    c_ref, a_ref = O.nf4_quantize(Wnew.astype(np.float32))
    assert np.array_equal(c, c_ref) and np.array_equal(a, a_ref)
    assert len(np.unique(c)) >= 12  # the merged weight exercises most levels
    assert np.array_equal(a, np.abs(Wnew).reshape(out, 2, 64).max(axis=2).astype(np.float32))


def test_merge_general_within_quantisation_error():
    L, Wq, Pq, B = _tiny(seed=8, out=64, inp=256)
    s = 1.0
    Wm = O.loqt_merge_f64(Wq, Pq, B, s)
    c, a = O.loqt_merge_requant(Wq, Pq, B, s)
    err = np.abs(O.nf4_dequantize_f64(c, a) - Wm)
    bound = 0.5 * (O.NF4_LEVELS[1] - O.NF4_LEVELS[0]) * np.repeat(a.astype(np.float64), 64, axis=1)
    assert np.all(err <= bound * (1 + 1e-6))
    assert np.array_equal(a, np.abs(Wm.astype(np.float32)).reshape(64, 4, 64).max(axis=2))
