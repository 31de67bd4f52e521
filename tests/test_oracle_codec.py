"""Pins for the oracle's NF4 codec (paper sec. 5.1): none of these re-types the
oracle's own formula; each checks it against the definition in rational arithmetic,
a closed form, or an invariant that the definition implies."""
from fractions import Fraction

import numpy as np
import pytest
from scipy.stats import norm

from oracle import loqt_oracle as O

Q = O.NF4_LEVELS


def test_levels_are_normal_quantiles():
    # Sec. 5.1: the levels are quantiles of the normal distribution; construction
    # published with the NF4 data type: 8 positive and 7 negative quantiles at equal
    # probability steps from an offset of (1/2)(1 - 1/32 + 1 - 1/30), plus an exact 0,
    # normalised to [-1, 1].
    off = 0.5 * ((1 - 1 / 32) + (1 - 1 / 30))
    pos = norm.ppf(np.linspace(off, 0.5, 9)[:-1])
    neg = -norm.ppf(np.linspace(off, 0.5, 8)[:-1])
    v = np.sort(np.concatenate([pos, [0.0], neg]))
    v /= np.abs(v).max()
    assert np.abs(v - Q).max() < 5e-7


def test_levels_structure():
    assert Q.shape == (16,)
    assert np.all(np.diff(Q) > 0)
    assert Q[0] == -1.0 and Q[7] == 0.0 and Q[15] == 1.0
    assert np.all(Q.astype(np.float32).astype(np.float64) == Q)  # fp32-representable
    assert (Q < 0).sum() == 7 and (Q > 0).sum() == 8  # asymmetric
    gaps = np.diff(Q)
    assert gaps.argmax() == 0 and abs(gaps[0] - 0.3038072) < 1e-7
    assert abs(gaps[14] - 0.2770432) < 1e-7


def test_midpoint_products_exact_in_fp64():
    # the exactness claim behind the threshold form
    rng = np.random.default_rng(1)
    ms = rng.standard_normal(200).astype(np.float32)
    ms = np.abs(np.concatenate([ms, np.float32([1e-30, 3e38, 2.0 ** -126, 1.1754942e-38])]))
    for j in range(15):
        m2 = Q[j] + Q[j + 1]
        assert Fraction(m2) == Fraction(Q[j]) + Fraction(Q[j + 1])
        for m in ms:
            assert Fraction(float(m2 * np.float64(m))) == Fraction(m2) * Fraction(float(m))


def _brute_codes(w_row):
    """argmin_i |w/M - q_i| in rational arithmetic, ties to the lower index."""
    out = []
    for b in range(0, len(w_row), 64):
        blk = [Fraction(float(v)) for v in w_row[b:b + 64]]
        M = max(abs(v) for v in blk)
        for v in blk:
            if M == 0:
                out.append(7)
                continue
            t = v / M
            best, bi = None, None
            for i in range(16):
                d = abs(t - Fraction(float(Q[i])))
                if best is None or d < best:
                    best, bi = d, i
            out.append(bi)
    return np.array(out, dtype=np.uint8)


@pytest.mark.parametrize("cols", [64, 128, 100, 21, 1])
def test_codes_equal_rational_argmin(cols):
    rng = np.random.default_rng(cols)
    w = (rng.standard_normal((3, cols)) * 0.02).astype(np.float32)
    w[1, : min(cols, 64)] *= np.float32(1e-20)  # tiny block
    codes, absmax = O.nf4_quantize(w)
    assert codes.shape == (3, cols) and absmax.shape == (3, -(-cols // 64))
    for i in range(3):
        assert np.array_equal(codes[i], _brute_codes(w[i]))
        for b in range(absmax.shape[1]):
            assert absmax[i, b] == np.abs(w[i, 64 * b:64 * b + 64]).max()


def test_exact_ties_go_to_lower_index():
    # absmax = 2^k makes (q_j + q_{j+1})/2 * absmax representable when the sum is:
    # build w exactly on each midpoint that is representable in fp32.
    for k in (-3, 0, 5):
        M = np.float32(2.0 ** k)
        ws, want = [M], [15]
        for j in range(15):
            mid = (Fraction(float(Q[j])) + Fraction(float(Q[j + 1]))) / 2 * Fraction(float(M))
            f = np.float32(float(mid))
            if Fraction(float(f)) == mid:  # exactly representable: a true tie
                ws.append(f)
                want.append(j)
                up = np.nextafter(f, np.float32(np.inf), dtype=np.float32)
                ws.append(up)
                want.append(j + 1)
        assert len(ws) > 10  # several midpoints are representable
        w = np.zeros((1, 64), dtype=np.float32)
        w[0, : len(ws)] = ws
        want = want + [7] * (64 - len(want))
        codes, absmax = O.nf4_quantize(w)
        assert absmax[0, 0] == M
        assert codes[0].tolist() == want


def test_absmax_element_and_zero_block():
    rng = np.random.default_rng(3)
    w = rng.standard_normal((4, 256)).astype(np.float32)
    w[2, 64:128] = 0.0
    w[3, 0:64] = -np.abs(w[3, 0:64])  # block whose extreme is negative
    codes, absmax = O.nf4_quantize(w)
    deq = O.nf4_dequantize_f32(codes, absmax)
    for i in range(4):
        for b in range(4):
            blk = w[i, 64 * b:64 * b + 64]
            if absmax[i, b] == 0:
                assert np.all(codes[i, 64 * b:64 * b + 64] == 7)
                assert np.all(deq[i, 64 * b:64 * b + 64] == 0.0)
                continue
            a = np.abs(blk).argmax()
            assert codes[i, 64 * b + a] == (15 if blk[a] > 0 else 0)
            assert deq[i, 64 * b + a] == blk[a]  # +-absmax returned exactly


def test_round_trip_bound_and_local_gap():
    rng = np.random.default_rng(4)
    w = (rng.standard_normal((64, 512)) * 0.02).astype(np.float32)
    codes, absmax = O.nf4_quantize(w)
    deq = O.nf4_dequantize_f64(codes, absmax)
    scale = np.repeat(absmax.astype(np.float64), 64, axis=1)
    err = np.abs(w.astype(np.float64) - deq)
    assert np.all(err <= 0.5 * (Q[1] - Q[0]) * scale)  # half the widest gap
    # tighter: at most half of the larger gap adjacent to the chosen level
    gaps = np.diff(Q)
    left = np.concatenate([[0.0], gaps])[codes]
    right = np.concatenate([gaps, [0.0]])[codes]
    assert np.all(err <= 0.5 * np.maximum(left, right) * scale * (1 + 1e-15))


def test_idempotent_scale_equivariant_asymmetric():
    rng = np.random.default_rng(5)
    w = (rng.standard_normal((8, 192)) * 0.02).astype(np.float32)
    c1, a1 = O.nf4_quantize(w)
    c2, a2 = O.nf4_quantize(O.nf4_dequantize_f32(c1, a1))
    assert np.array_equal(c1, c2) and np.array_equal(a1, a2)
    for k in (-7, 9):
        c3, a3 = O.nf4_quantize(w * np.float32(2.0 ** k))
        assert np.array_equal(c1, c3) and np.array_equal(a3, a1 * np.float32(2.0 ** k))
    cneg, aneg = O.nf4_quantize(-w)
    assert np.array_equal(aneg, a1)
    assert not np.array_equal(cneg, 15 - c1)  # 7 negative vs 8 positive levels


def test_dequant_outputs_and_bf16_rounding():
    codes = np.arange(16, dtype=np.uint8).reshape(1, 16)
    absmax = np.float32([[0.0371]])
    f64 = O.nf4_dequantize_f64(codes, absmax)
    for i in range(16):
        assert Fraction(float(f64[0, i])) == Fraction(float(Q[i])) * Fraction(float(absmax[0, 0]))
    f32 = O.nf4_dequantize_f32(codes, absmax)
    assert f32.dtype == np.float32 and np.all(np.abs(f32 - f64) <= np.abs(f64) * 2.0 ** -24)
    # bf16: RNE cases with known answers
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e-5, 0.0], dtype=np.float32)
    # 1.00390625 = 1 + 2^-8: tie -> even (1.0); 1.01171875 = 1 + 3*2^-8: tie -> 1 + 2^-6
    bits = O.f32_to_bf16_rne(x)
    assert bits[0] == 0x3F80 and bits[1] == 0x3F80 and bits[2] == 0x3F82 and bits[4] == 0
    back = O.bf16_to_f64(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    b16 = O.nf4_dequantize_bf16(codes, absmax)
    assert np.all(np.abs(O.bf16_to_f64(b16) - f64) <= np.abs(f64) * 2.0 ** -8)


@pytest.mark.parametrize("cols,ld", [(128, 128), (100, 128), (21, 64), (5461, 5504)])
def test_pack_layout_and_memory(cols, ld):
    rng = np.random.default_rng(6)
    w = rng.standard_normal((5, cols)).astype(np.float32)
    codes, absmax = O.nf4_quantize(w)
    packed, am = O.pack_nf4(codes, absmax, ld)
    assert packed.shape == (5, ld // 2) and am.shape == (5, ld // 64)
    # 0.5 byte per code + 4 bytes per 64 (the 4-bit term of the paper's memory table)
    assert packed.nbytes + am.nbytes == 5 * ld * 0.5625
    assert (packed[2, 0] >> 4) == codes[2, 0]
    if cols > 1:
        assert (packed[2, 0] & 0xF) == codes[2, 1]
    c2, a2 = O.unpack_nf4(packed, am, cols)
    assert np.array_equal(c2, codes) and np.array_equal(a2, absmax)
    full = np.empty((5, ld), np.uint8)
    full[:, 0::2] = packed >> 4
    full[:, 1::2] = packed & 0xF
    assert np.all(full[:, cols:] == 7)
    assert np.all(am[:, -(-cols // 64):] == 0)


def test_decision_points_are_isolated_in_sixteenth_buckets():
    """Geometry of the level table that a bucketed encoder may rely on (sec. 5.1): cut u = w/M into
    buckets of width 1/16 with edges at odd multiples of 1/32.  Every bucket, widened by a guard of
    1e-4 on both sides, holds at most one decision point (q_j + q_{j+1})/2, and no decision point
    lies within 3e-3 of an edge; so 'code at the left edge, plus one exact comparison against the
    next decision point' is the argmin for every element that lands in the bucket."""
    q = [Fraction(float(v)) for v in O.NF4_LEVELS]
    mids = [(q[j] + q[j + 1]) / 2 for j in range(15)]
    assert min(b - a for a, b in zip(mids, mids[1:])) > Fraction(1, 16)
    guard = Fraction(1, 10000)
    for k in range(0, 33):
        left, right = Fraction(2 * k - 33, 32), Fraction(2 * k - 31, 32)
        inside = [m for m in mids if left - guard <= m <= right + guard]
        assert len(inside) <= 1
        for m in mids:
            assert abs(m - left) > Fraction(3, 1000) and abs(m - right) > Fraction(3, 1000)
    # brute force: bucket rule == argmin on a dense grid of u (M = 1), ties included
    for num in range(-4096, 4097):
        u = Fraction(num, 4096)
        k = round(16 * u) + 16            # any rounding of ties works: edges are guard-banded
        left = Fraction(2 * k - 33, 32)
        c0 = sum(1 for m in mids if m < left - guard)
        code = c0 + (1 if c0 < 15 and u > mids[c0] else 0)
        assert code == sum(1 for m in mids if u > m)


def test_single_precision_decision_is_exact_outside_its_guard_band():
    """An encoder may take the one deciding comparison in single precision: with th32 = fl32(fl32(mid_j) * M) and
    d = fl32(w - th32), the sign of d is the sign of the exact w - mid_j M whenever |d| > 2^-22 M (th32 is within
    2^-23 M of the exact threshold, d within 2^-24 |d| of w - th32), provided M is a normal number far from the
    ends of the range.  Checked here in exact rational arithmetic on the values where it could fail: every fp32
    neighbour of every threshold, at scales across the allowed range, and random elements; and the share of
    random elements that fall inside the guard band (they take the exact path) is of the order 1e-6."""
    q = [Fraction(float(v)) for v in O.NF4_LEVELS]
    mids = [(q[j] + q[j + 1]) / 2 for j in range(15)]
    mids32 = np.array([float(m) for m in mids], dtype=np.float32)  # fl32(mid): float(m) is exact (29 bits), then RNE
    rng = np.random.default_rng(3)
    scales = [np.float32(2.0) ** e for e in (-100, -60, -24, -7, 0, 5, 40, 100)]
    scales += list((rng.uniform(1.0, 2.0, 6).astype(np.float32)) * np.float32(2.0) ** rng.integers(-90, 90, 6))
    checked = 0
    for M in scales:
        M = np.float32(M)
        guard = np.float32(M * np.float32(2.0 ** -22))
        for j in range(15):
            th32 = np.float32(mids32[j] * M)
            exact_th = mids[j] * Fraction(float(M))
            # the fp32 values around the threshold, a few steps to each side
            w = th32
            cand = [w]
            lo = hi = w
            for _ in range(40):
                lo = np.nextafter(lo, np.float32(-np.inf), dtype=np.float32)
                hi = np.nextafter(hi, np.float32(np.inf), dtype=np.float32)
                cand += [lo, hi]
            for w in cand:
                d = np.float32(w - th32)
                if abs(d) > guard:
                    assert (d > 0) == (Fraction(float(w)) > exact_th), (float(M), j, float(w))
                    checked += 1
    assert checked > 1000
    # random elements of random blocks: outside the guard band the fast decision equals the exact one
    near = total = 0
    for _ in range(40):
        M = np.float32(rng.uniform(0.5, 2.0) * 2.0 ** rng.integers(-30, 30))
        w = (rng.uniform(-1, 1, 20000) * M).astype(np.float32)
        for j in range(15):
            th32 = np.float32(mids32[j] * M)
            d = (w - th32).astype(np.float32)
            sure = np.abs(d) > np.float32(M * np.float32(2.0 ** -22))
            # inside the band anything may happen (those elements take the exact path); outside, compare in float64,
            # which decides correctly there (|w - mid M| > 2^-23 M, and mid M is exact in float64)
            ref = w.astype(np.float64) > float(mids[j]) * float(M)
            assert np.array_equal((d > 0)[sure], ref[sure])
            near += int((~sure).sum())
            total += w.size
    assert near / total < 2e-5
