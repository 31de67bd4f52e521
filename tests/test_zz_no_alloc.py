"""The allocation-free entry point loqt_absmax_dq_compress_static (for callers that cannot allocate: HIP graph
capture, serving loops) against loqt_absmax_dq_compress, which takes a caller's workspace: same codes, block
constants and mean, bit for bit, on two calls in a row, the second with a smaller input (the static scratch keeps
the first call's partial sums); sizes beyond the fixed scratch are refused on the host."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _scales(n, seed):
    rng = np.random.default_rng(seed)
    return (np.abs(rng.normal(0.0, 0.02, n)) * 3.0 + 1e-3).astype(np.float32)


def _static(L, a_dev):
    n = a_dev.numel()
    codes = torch.full((n,), 0xAA, dtype=torch.uint8, device="cuda")
    c1 = torch.full(((n + 255) // 256,), -1.0, dtype=torch.float32, device="cuda")
    mean = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    st = L.lib.loqt_absmax_dq_compress_static(a_dev.data_ptr(), n, codes.data_ptr(), c1.data_ptr(), mean.data_ptr(),
                                              torch.cuda.current_stream().cuda_stream)
    assert st == 0, L.STATUS_NAMES.get(st, st)
    return codes, c1, mean


def test_static_matches_workspace_variant_twice_in_a_row():
    from paper_2405_16528_amd import binding as L
    # 11008 x 4096 / 64 scales + a ragged tail (173 partial sums), then a much smaller input (3 partial sums)
    for n, seed in ((11008 * 4096 // 64 + 37, 1), (9001, 2)):
        a = torch.from_numpy(_scales(n, seed)).cuda()
        ref_codes, ref_c1, ref_mean = L.loqt_absmax_dq_compress(a)
        codes, c1, mean = _static(L, a)
        torch.cuda.synchronize()
        assert torch.equal(mean, ref_mean), (n, float(mean), float(ref_mean))
        assert torch.equal(c1, ref_c1), n
        assert torch.equal(codes, ref_codes), n


def test_static_rejects_sizes_beyond_its_scratch():
    from paper_2405_16528_amd import binding as L
    limit = int(L.lib.loqt_absmax_dq_static_max_n())
    assert limit == 1 << 25
    a = torch.zeros(16, dtype=torch.float32, device="cuda")
    out = torch.zeros(16, dtype=torch.uint8, device="cuda")
    f = torch.zeros(1, dtype=torch.float32, device="cuda")
    # the size is checked on the host before anything is launched or any buffer is touched
    st = L.lib.loqt_absmax_dq_compress_static(a.data_ptr(), C.c_int64(limit + 1), out.data_ptr(), f.data_ptr(),
                                              f.data_ptr(), None)
    assert L.STATUS_NAMES[st] == "LOQT_STATIC_SCRATCH_TOO_SMALL"
    st = L.lib.loqt_absmax_dq_compress_static(a.data_ptr(), C.c_int64(0), out.data_ptr(), f.data_ptr(), f.data_ptr(), None)
    assert L.STATUS_NAMES[st] == "LOQT_BAD_SHAPE"
    st = L.lib.loqt_absmax_dq_compress_static(None, C.c_int64(16), out.data_ptr(), f.data_ptr(), f.data_ptr(), None)
    assert L.STATUS_NAMES[st] == "LOQT_INVALID_ARG"
