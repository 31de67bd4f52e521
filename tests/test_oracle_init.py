"""Pins for the oracle's error-compensated initialisation (Alg. 2 lines 5-11, sec. 2.5):
closed forms, least-squares optimality checked without the pseudo-inverse, special cases and the
invariants a wrong sign, a dropped scale or a transposed operand would break."""
import numpy as np
import pytest

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth


def _case(out, inp, r, seed=0):
    rng = synth.rng_for(seed, "init", str(out), str(inp), str(r))
    W = synth.normal_f32(rng, (out, inp), 0.02)
    P = synth.orthonormal_f32(rng, out, r)
    return W, P


def _objective(W, P, codes, absmax, B, s):
    return float(np.linalg.norm(O.nf4_dequantize_f64(codes, absmax) + s * (P.astype(np.float64) @ B)
                                - W.astype(np.float64)))


def test_first_step_is_plain_quantisation_plus_least_squares():
    W, P = _case(96, 192, 24)
    s = 0.5
    codes, absmax, B, hist = O.loqt_init_compensate(W, P, s, 1)
    c0, a0 = O.nf4_quantize(W)  # Alg. 2 line 8 with W_hat = W
    assert np.array_equal(codes, c0) and np.array_equal(absmax, a0)
    # normal equations, no pseudo-inverse involved: the residual is orthogonal to range(P)
    Pd = P.astype(np.float64)
    R = W.astype(np.float64) - O.nf4_dequantize_f64(codes, absmax) - s * (Pd @ B)
    assert np.linalg.norm(Pd.T @ R) <= 1e-12 * np.linalg.norm(R) * np.linalg.norm(Pd)
    assert hist[0] == pytest.approx(np.linalg.norm(R), rel=1e-12)
    # any perturbation of B makes the fit worse; B = 0 (no compensation) is worse too
    rng = np.random.default_rng(5)
    base = _objective(W, P, codes, absmax, B, s)
    for _ in range(5):
        D = rng.standard_normal(B.shape) * 1e-4
        assert _objective(W, P, codes, absmax, B + D, s) > base
    assert base < _objective(W, P, codes, absmax, np.zeros_like(B), s)
    # the opposite sign (B = P^+(Q - W)) would be worse than no compensation at all
    assert _objective(W, P, codes, absmax, -B, s) > _objective(W, P, codes, absmax, np.zeros_like(B), s)


def test_pseudo_inverse_not_transpose():
    """P with columns of norm 2: P^+ = P^T / 4.  Closed form for the least-squares B."""
    W, P = _case(64, 128, 8, seed=1)
    P2 = (2.0 * P).astype(np.float32)
    codes, absmax, B, _ = O.loqt_init_compensate(W, P2, 1.0, 1)
    E = W.astype(np.float64) - O.nf4_dequantize_f64(codes, absmax)
    G = P2.astype(np.float64).T @ P2.astype(np.float64)
    B_ref = np.linalg.solve(G, P2.astype(np.float64).T @ E)
    assert np.allclose(B, B_ref, rtol=1e-9, atol=1e-15)
    assert np.allclose(B, P2.astype(np.float64).T @ E / 4.0, rtol=1e-5, atol=1e-12)


def test_square_orthogonal_projection_removes_the_error_completely():
    """r = out: range(P) is everything, so Q + s P B = W after every step."""
    W, P = _case(64, 128, 64, seed=2)
    for iters in (1, 3):
        codes, absmax, B, hist = O.loqt_init_compensate(W, P, 0.25, iters)
        assert hist[-1] <= 1e-6 * np.linalg.norm(W)  # P is orthogonal to fp32 accuracy only
        assert _objective(W, P, codes, absmax, B, 0.25) == pytest.approx(hist[-1], rel=1e-9, abs=1e-15)


def test_representable_weight_is_a_fixed_point():
    _, P = _case(64, 192, 16, seed=3)
    rng = np.random.default_rng(3)
    c0 = rng.integers(0, 16, size=(64, 192)).astype(np.uint8)
    c0[:, ::64] = 15                                     # every block attains its absmax
    a0 = np.full((64, 3), 2.0 ** -6, dtype=np.float32)   # power of two: level * absmax is exact in fp32
    W = O.nf4_dequantize_f32(c0, a0)
    assert np.array_equal(W.astype(np.float64), O.nf4_dequantize_f64(c0, a0))
    codes, absmax, B, hist = O.loqt_init_compensate(W, P, 1.0, 3)
    assert np.array_equal(codes, c0) and np.array_equal(absmax, a0)
    assert np.all(B == 0.0) and hist == [0.0, 0.0, 0.0]


def test_compensation_reduces_the_error_and_keeps_reducing_it():
    """sec. 2.5: the loop improves the alignment of Q + P B with W; on the synthetic recipe the
    objective falls at every step and ends well below the plain quantisation error."""
    W, P = _case(256, 512, 64, seed=4)
    codes, absmax, B, hist = O.loqt_init_compensate(W, P, 1.0, 5)
    plain = float(np.linalg.norm(O.nf4_dequantize_f64(*O.nf4_quantize(W)) - W.astype(np.float64)))
    assert all(b <= a * (1 + 1e-12) for a, b in zip(hist, hist[1:]))
    # projecting out r of `out` directions removes about r/out of the squared error
    assert hist[0] < plain * np.sqrt(1 - 0.8 * 64 / 256)
    assert hist[-1] < hist[0]
    assert _objective(W, P, codes, absmax, B, 1.0) == pytest.approx(hist[-1], rel=1e-12)


def test_scale_and_warm_start_consistency():
    W, P = _case(128, 256, 32, seed=5)
    c1, a1, B1, h1 = O.loqt_init_compensate(W, P, 1.0, 3)
    c4, a4, B4, h4 = O.loqt_init_compensate(W, P, 0.25, 3)  # power of two: exact rescaling
    assert np.array_equal(c1, c4) and np.array_equal(a1, a4)
    assert np.allclose(B4, 4.0 * B1, rtol=1e-12, atol=0) and np.allclose(h1, h4, rtol=1e-12)
    # three steps = two steps, then one more from the B they produced
    _, _, B2, h2 = O.loqt_init_compensate(W, P, 1.0, 2)
    c3, a3, B3, h3 = O.loqt_init_compensate(W, P, 1.0, 1, B0=B2)
    assert np.array_equal(c3, c1) and np.array_equal(a3, a1) and np.array_equal(B3, B1)
    assert h2 == h1[:2] and h3 == h1[2:]


def test_the_box_line_taken_literally_does_not_descend():
    """Alg. 2 prints the update as B <- P^+(W_hat - Q_c) with W_hat = W - P B.  For orthonormal P that is the
    least-squares B minus the previous B: from the second iteration on it is the *increment* of the least-squares
    solution, not the solution.  Iterated literally, the stated objective |Q_c + P B - W| is not monotone (it goes
    back up on every second iteration) and ends well above the reading implemented (B = P^+(W - Q_c)), which is
    non-increasing.  Both loops written out here with the oracle's quantiser."""
    W, P = _case(128, 256, 32, seed=4)
    Wd, Pd = W.astype(np.float64), P.astype(np.float64)
    Pp = np.linalg.pinv(Pd)

    def objective(codes, absmax, B):
        return float(np.linalg.norm(O.nf4_dequantize_f64(codes, absmax) + Pd @ B - Wd))

    # the line as printed
    B = np.zeros((32, 256))
    W_hat = Wd.copy()
    literal = []
    for _ in range(5):
        codes, absmax = O.nf4_quantize(W_hat.astype(np.float32))
        B = Pp @ (W_hat - O.nf4_dequantize_f64(codes, absmax))
        W_hat = Wd - Pd @ B
        literal.append(objective(codes, absmax, B))
    # the least-squares reading (s = 1): the oracle's loop
    _, _, _, hist = O.loqt_init_compensate(W, P, 1.0, 5)
    assert all(b <= a * (1 + 1e-12) for a, b in zip(hist, hist[1:]))   # non-increasing
    assert hist[-1] < 0.9 * hist[0]
    assert literal[0] == pytest.approx(hist[0], rel=1e-9)              # the first iteration is the same (W_hat = W)
    assert literal[1] > literal[0] and literal[3] > literal[2]         # the literal form goes back up
    assert all(l > h * 1.05 for l, h in zip(literal[1:], hist[1:]))    # and stays above the least-squares loop
