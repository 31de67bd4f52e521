"""GPU parity of the double-quantised block scales (loqt_absmax_dq_compress / loqt_absmax_dq_expand) against the
oracle: codes, block constants and expanded scales bit for bit.  The mean is stored by the format, so the device's
fixed-order fp64 sum may differ from the oracle's by at most one fp32 step; the oracle is then given the device's
mean, as the format allows."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O

pytestmark = pytest.mark.gpu


def _scales(n, seed, sigma=0.02):
    rng = np.random.default_rng(seed)
    out = np.empty(n, dtype=np.float32)
    step = 1 << 16
    for i in range(0, n, step):
        m = min(step, n - i)
        out[i:i + m] = np.abs(rng.normal(0, sigma, (m, 64))).max(axis=1).astype(np.float32)
    return out


@pytest.mark.parametrize("n", [1, 63, 256, 257, 4097, 10000, 4096 * 4096 // 64, 11008 * 4096 // 64 + 3])
def test_compress_expand_parity(n):
    from paper_2405_16528_amd import binding as L
    a = _scales(n, n)
    if n >= 10000:  # a block of equal scales and a block holding a zero scale
        a[512:768] = a[512]
        a[1024] = 0.0
    dev = torch.from_numpy(a).cuda()
    codes, c1, mean = L.loqt_absmax_dq_compress(dev)
    torch.cuda.synchronize()
    mean_h = mean.cpu().numpy()[0]
    _, _, mean_ref = O.absmax_dq_compress(a)
    assert abs(float(mean_h) - float(mean_ref)) <= np.spacing(np.float32(mean_ref))
    codes_ref, c1_ref, _ = O.absmax_dq_compress(a, mean=mean_h)
    assert np.array_equal(c1.cpu().numpy(), c1_ref)
    assert np.array_equal(codes.cpu().numpy(), codes_ref)
    back = L.loqt_absmax_dq_expand(codes, c1, mean)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy(), O.absmax_dq_expand(codes_ref, c1_ref, mean_h))
    # a second run gives the same bits (fixed-order sum)
    codes2, c12, mean2 = L.loqt_absmax_dq_compress(dev)
    assert torch.equal(codes2, codes) and torch.equal(c12, c1) and torch.equal(mean2, mean)


def test_every_code_expands_exactly():
    from paper_2405_16528_amd import binding as L
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F] * 3, dtype=np.uint8)
    c1 = np.float32([0.013, 1.0, 7.5e-4])[: (codes.size + 255) // 256]
    mean = np.float32([0.0517])
    got = L.loqt_absmax_dq_expand(torch.from_numpy(codes).cuda(), torch.from_numpy(c1).cuda(), torch.from_numpy(mean).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), O.absmax_dq_expand(codes, c1, mean[0]))


def test_encoder_on_ties_and_boundaries():
    """Scales built so that fl32(d / c1) * 448 lands on representable values, on midpoints between them and next to
    both: with mean 0 and c1 = 448 * 2^k the scaled value is d * 2^-k exactly."""
    from paper_2405_16528_amd import binding as L
    pos = np.array([c for c in range(0x7F)], dtype=np.uint8)
    vals = O.e4m3_decode(pos).astype(np.float64)
    mid = (vals[:-1] + vals[1:]) / 2
    u = np.concatenate([vals, mid, np.nextafter(mid.astype(np.float32), np.float32(1e9)).astype(np.float64),
                        np.nextafter(mid.astype(np.float32), np.float32(0)).astype(np.float64)]).astype(np.float32)
    # the format subtracts the mean: place the values symmetrically so that the mean is exactly 0
    a = np.concatenate([u, -u]).astype(np.float32) * np.float32(2.0 ** -3)
    a = np.concatenate([a, np.float32([448 * 2.0 ** -3, -448 * 2.0 ** -3])])
    pad = (-a.size) % 256
    a = np.concatenate([a, np.zeros(pad, dtype=np.float32)])
    # every block must contain +-448 * 2^-3 so that c1 is the same everywhere: interleave
    nb = a.size // 256
    blocks = a.reshape(nb, 256).copy()
    blocks[:, 0] = np.float32(448 * 2.0 ** -3)
    blocks[:, 1] = np.float32(-448 * 2.0 ** -3)
    a = blocks.reshape(-1)
    a = np.concatenate([a, -a])  # mean exactly zero again
    dev = torch.from_numpy(a).cuda()
    codes, c1, mean = L.loqt_absmax_dq_compress(dev)
    torch.cuda.synchronize()
    assert float(mean.cpu()[0]) == 0.0
    codes_ref, c1_ref, _ = O.absmax_dq_compress(a, mean=np.float32(0))
    assert np.array_equal(c1.cpu().numpy(), c1_ref) and np.array_equal(codes.cpu().numpy(), codes_ref)
