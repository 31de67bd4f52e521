"""Pins of the oracle's double-quantised block scales (paper sec. 2.4: the quantisation state is itself
quantised again).  The paper gives no format (parity unpinned by the paper); what is pinned here is the oracle's
arithmetic for the reading it states: the 8-bit float against a library cast, round-trip bounds, closed forms."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O


def test_e4m3_decode_matches_library_cast_on_every_code():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).float().numpy()
    mine = O.e4m3_decode(codes)
    nan = np.isnan(lib)
    assert np.array_equal(nan, np.isnan(mine)) and nan.sum() == 2  # 0x7f, 0xff
    assert np.array_equal(lib[~nan], mine[~nan])
    # closed forms: largest value, smallest normal, smallest subnormal, one
    assert mine[0x7E] == 448.0 and mine[0x08] == 2.0 ** -6 and mine[0x01] == 2.0 ** -9 and mine[0x38] == 1.0
    assert mine[0x80] == 0.0 and np.signbit(mine[0x80])


def test_e4m3_encode_is_nearest_ties_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 120, 200000), rng.normal(0, 1, 200000), rng.normal(0, 0.01, 100000)]).astype(np.float32)
    x = np.clip(x, -448, 448)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(O.e4m3_encode(x), lib)
    # every representable value encodes to itself; every midpoint goes to the even mantissa
    pos = np.array([c for c in range(0x7F)], dtype=np.uint8)
    vals = O.e4m3_decode(pos)
    assert np.array_equal(O.e4m3_encode(vals), pos)
    assert np.array_equal(O.e4m3_encode(-vals), pos | 0x80)
    mid = ((vals[:-1].astype(np.float64) + vals[1:]) / 2).astype(np.float32)  # exact in fp32
    enc = O.e4m3_encode(mid)
    want = np.where(pos[:-1] % 2 == 0, pos[:-1], pos[1:])
    assert np.array_equal(enc, want)
    # just off a midpoint: the nearer neighbour
    assert np.array_equal(O.e4m3_encode(np.nextafter(mid, np.float32(np.inf))), pos[1:])
    assert np.array_equal(O.e4m3_encode(np.nextafter(mid[1:], np.float32(0))), pos[1:-1])
    # saturation
    assert O.e4m3_encode(np.float32([1e9, -1e9, 448.0, 464.0])).tolist() == [0x7E, 0xFE, 0x7E, 0x7E]


def _scales(n, seed):
    rng = np.random.default_rng(seed)
    # block scales of N(0, 0.02) weights: maxima of 64 half-normals
    w = rng.normal(0, 0.02, (n, 64)).astype(np.float32)
    return np.abs(w).max(axis=1)


@pytest.mark.parametrize("n", [1, 255, 256, 257, 1000, 4096 * 64])
def test_round_trip_bound(n):
    a = _scales(n, n)
    codes, c1, mean = O.absmax_dq_compress(a)
    assert codes.shape == (n,) and c1.shape == ((n + 255) // 256,) and mean.dtype == np.float32
    b = O.absmax_dq_expand(codes, c1, mean)
    # half an E4M3 step at the top of the range is 16 of 448, i.e. c1 / 28, plus fp32 rounding
    bound = np.repeat(c1, 256)[:n].astype(np.float64) / 28 * (1 + 1e-5) + 1e-7 * np.abs(a)
    assert np.all(np.abs(b.astype(np.float64) - a) <= bound)
    # per element it is relative: half a step of a 3-bit mantissa is 2^-4 of |M - mean| (plus the subnormal
    # step of the format, 2^-9 of 448ths of c1, and fp32 rounding)
    d = np.abs(a.astype(np.float64) - float(mean))
    assert np.all(np.abs(b.astype(np.float64) - a) <= d / 16 * (1 + 1e-5) + np.repeat(c1, 256)[:n] * 2.0 ** -9 / 448 + 1e-7 * np.abs(a))


def test_constant_scales_survive_exactly():
    a = np.full(1000, np.float32(0.0537), dtype=np.float32)
    codes, c1, mean = O.absmax_dq_compress(a)
    assert mean == a[0] and not c1.any() and not (codes & 0x7F).any()
    assert np.array_equal(O.absmax_dq_expand(codes, c1, mean), a)


def test_power_of_two_scaling_and_block_locality():
    a = _scales(2000, 7)
    codes, c1, mean = O.absmax_dq_compress(a)
    for k in (-20, 3, 40):
        f = np.float32(2.0 ** k)
        codes2, c12, mean2 = O.absmax_dq_compress(a * f)
        assert np.array_equal(codes2, codes) and np.array_equal(c12, c1 * f) and mean2 == mean * f
    # with the mean fixed, a block's codes depend on that block alone
    a2 = a.copy()
    a2[300:400] *= np.float32(1.5)
    codes3, c13, _ = O.absmax_dq_compress(a2, mean=mean)
    blk = slice(256, 512)
    assert np.array_equal(np.delete(codes3, np.r_[blk]), np.delete(codes, np.r_[blk]))
    assert np.array_equal(np.delete(c13, 1), np.delete(c1, 1))


def test_extreme_of_a_block_takes_the_largest_code():
    a = _scales(512, 3)
    codes, c1, mean = O.absmax_dq_compress(a)
    d = (a - mean).astype(np.float32)
    for b in range(2):
        i = b * 256 + int(np.argmax(np.abs(d[b * 256:(b + 1) * 256])))
        assert (codes[i] & 0x7F) == 0x7E and bool(codes[i] & 0x80) == bool(d[i] < 0)
        assert c1[b] == np.abs(d[i])


def test_storage_per_weight():
    # 4 bits per weight, 8 bits per 64 weights, 32 bits per 256 x 64 weights (sec. 2.4 / the memory table counts
    # the weights at 4 bit; the scales are the remainder)
    n = 4096 * 4096
    codes, c1, _ = O.absmax_dq_compress(np.ones(n // 64, dtype=np.float32))
    total = n / 2 + codes.nbytes + c1.nbytes + 4
    assert abs(total / n - (0.5 + 1 / 64 + 4 / (64 * 256))) < 1e-6
