"""GPU parity of nf4_quantize / nf4_dequantize against the oracle: bit-exact codes, absmax
and dequantised values, including padding, short blocks, ties and zero blocks."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth

pytestmark = pytest.mark.gpu


def _L():
    from paper_2405_16528_amd import binding
    return binding


def _quantize_both(w, ld_w=None, ld_q=None):
    from tests import gpu_util as G
    L = _L()
    rows, cols = w.shape
    ld_w = ld_w or G.rup(cols, 4)
    buf = np.full((rows, ld_w), np.float32(123.0))  # pitch padding must be ignored
    buf[:, :cols] = w
    wd = torch.from_numpy(buf).cuda()
    q = L.NF4Tensor.empty(rows, cols, ld_q)
    q.codes.fill_(0xAB)
    q.absmax.fill_(-1.0)
    L.nf4_quantize(wd, q, cols=cols)
    torch.cuda.synchronize()
    c_ref, a_ref = O.nf4_quantize(w)
    return q, c_ref, a_ref


@pytest.mark.parametrize("rows,cols,ld_q", [(4, 64, None), (37, 1000, 1024), (3, 5461, 5504), (129, 4096, None),
                                            (1, 21, 128), (2048, 2048, None)])
def test_quantize_bit_exact(rows, cols, ld_q):
    from tests import gpu_util as G
    w = synth.normal_f32(synth.rng_for(0, "codec", rows, cols), (rows, cols), 0.02)
    q, c_ref, a_ref = _quantize_both(w, ld_q=ld_q)
    c, a, packed, am = G.nf4_host(q)
    assert np.array_equal(a, a_ref)
    assert np.array_equal(c, c_ref)
    p_ref, am_ref = O.pack_nf4(c_ref, a_ref, q.ld)  # padding nibbles 7, padding absmax 0
    assert np.array_equal(packed, p_ref) and np.array_equal(am, am_ref)


def test_quantize_adversarial():
    from tests import gpu_util as G
    rng = synth.rng_for(1, "adversarial")
    Q = O.NF4_LEVELS
    rows = []
    # (a) values on and next to every midpoint, for several scales, normal and tiny
    for k in (-140, -126, -30, -3, 0, 7, 100):
        M = np.float32(2.0 ** k)
        vals = [M, -M]
        for j in range(15):
            mid = np.float32((Q[j] + Q[j + 1]) * 0.5 * float(M))
            for d in (-2, -1, 0, 1, 2):
                v = mid
                for _ in range(abs(d)):
                    v = np.nextafter(v, np.float32(np.inf if d > 0 else -np.inf), dtype=np.float32)
                vals.append(v)
        row = np.zeros(128, dtype=np.float32)
        row[: len(vals)] = vals[:128]
        row[64] = M * np.float32(0.999)
        rows.append(row)
    # (b) a non power-of-two absmax with values near midpoints in fp32
    for M in (0.0371, 1.7, 3.0e-5):
        M = np.float32(M)
        vals = [M]
        for j in range(15):
            mid = np.float32(np.float64(Q[j] + Q[j + 1]) * 0.5 * np.float64(M))
            vals += [np.nextafter(mid, np.float32(-np.inf), dtype=np.float32), mid,
                     np.nextafter(mid, np.float32(np.inf), dtype=np.float32)]
        row = np.zeros(128, dtype=np.float32)
        row[: len(vals)] = vals
        row[64:] = rng.standard_normal(64).astype(np.float32) * M
        rows.append(row)
    # (c) zero block, negative extreme, denormals
    row = np.zeros(128, dtype=np.float32)
    row[64:] = -np.abs(rng.standard_normal(64).astype(np.float32))
    rows.append(row)
    rows.append((rng.standard_normal(128) * 1e-41).astype(np.float32))
    w = np.stack(rows)
    q, c_ref, a_ref = _quantize_both(w)
    c, a, _, _ = G.nf4_host(q)
    assert np.array_equal(a, a_ref)
    bad = np.argwhere(c != c_ref)
    assert bad.size == 0, f"first mismatches {bad[:5]}"


@pytest.mark.parametrize("rows,cols,ld_q", [(5, 64, None), (33, 1000, 1024), (3, 5461, 5504), (300, 2048, None)])
def test_dequantize_bit_exact(rows, cols, ld_q):
    from tests import gpu_util as G
    L = _L()
    w = synth.normal_f32(synth.rng_for(2, "deq", rows, cols), (rows, cols), 0.02)
    c_ref, a_ref = O.nf4_quantize(w)
    q = G.nf4_dev(c_ref, a_ref, ld_q)
    out32 = torch.full((rows, G.rup(cols, 4) + 4), 7.0, dtype=torch.float32, device="cuda")
    L.nf4_dequantize(q, out32[:, :cols])
    out16 = G.bf16_empty(rows, cols, G.rup(cols, 8) + 8, fill=7.0)
    L.nf4_dequantize(q, out16)
    torch.cuda.synchronize()
    got32 = out32.cpu().numpy()
    assert np.array_equal(got32[:, :cols].view(np.uint32), O.nf4_dequantize_f32(c_ref, a_ref).view(np.uint32))
    assert np.all(got32[:, cols:] == 7.0)  # nothing written past cols
    assert np.array_equal(G.bf16_host(out16), O.nf4_dequantize_bf16(c_ref, a_ref))


def test_round_trip_on_device_is_idempotent():
    from tests import gpu_util as G
    L = _L()
    w = synth.normal_f32(synth.rng_for(3, "idem"), (64, 1024), 0.02)
    wd = torch.from_numpy(w).cuda()
    q1 = L.nf4_quantize(wd)
    deq = torch.empty_like(wd)
    L.nf4_dequantize(q1, deq)
    q2 = L.nf4_quantize(deq)
    torch.cuda.synchronize()
    assert torch.equal(q1.codes, q2.codes) and torch.equal(q1.absmax, q2.absmax)
