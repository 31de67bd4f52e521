"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2405_16528_amd", "libloqt.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2405_16528_amd import build
        build.build(verbose=False)
    from paper_2405_16528_amd import binding
    return binding.lib


def test_every_declared_symbol_is_exported(lib):
    hdr = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                  if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(nf4_\w+|loqt_\w+)\s*\(", hdr))
    assert {"nf4_quantize", "nf4_dequantize", "loqt_linear_fwd", "loqt_linear_bwd", "loqt_merge_requant",
            "loqt_merge_requant_batched", "loqt_workspace_bytes", "loqt_status_string", "loqt_set_path",
            "loqt_init_compensate", "loqt_linear_fwd_right", "loqt_linear_bwd_right",
            "loqt_merge_requant_right", "loqt_merge_dense", "loqt_adam_step", "loqt_merge_schedule",
            "loqt_absmax_dq_workspace_bytes", "loqt_absmax_dq_compress", "loqt_absmax_dq_expand",
            "loqt_linear_fwd_nq", "loqt_linear_bwd_nq", "loqt_merge_nq", "loqt_linear_fwd_save",
            "loqt_linear_bwd_saved", "loqt_set_tile", "loqt_plan_product", "loqt_prepare",
            "loqt_merge_batched_workspace_bytes", "loqt_absmax_dq_compress_static", "loqt_timing_enable"} <= names
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in loqt.h but not exported"


def test_status_strings(lib):
    assert lib.loqt_status_string(0) == b"LOQT_OK"
    assert lib.loqt_status_string(4) == b"LOQT_WORKSPACE_TOO_SMALL"
    assert lib.loqt_status_string(99) == b"LOQT_UNKNOWN_STATUS"


def test_workspace_sizes(lib):
    from paper_2405_16528_amd import binding as L
    T, out, inp, r = 8192, 4096, 4096, 1024
    fwd = L.loqt_workspace_bytes(L.OP_FWD, T, out, inp, r)
    bwd = L.loqt_workspace_bytes(L.OP_BWD, T, out, inp, r)
    mrg = L.loqt_workspace_bytes(L.OP_MERGE, 0, out, inp, r)
    assert fwd >= T * r * 2 + out * inp * 2 + out * r * 2
    assert bwd >= T * r * 2 + inp * out * 2 + r * out * 2 + r * inp * 4
    assert mrg >= out * r * 2
    fr = L.loqt_workspace_bytes(L.OP_FWD_RIGHT, T, out, inp, r)
    br = L.loqt_workspace_bytes(L.OP_BWD_RIGHT, T, out, inp, r)
    mr = L.loqt_workspace_bytes(L.OP_MERGE_RIGHT, 0, out, inp, r)
    assert fr >= inp * r * 2 + out * inp * 2 and br >= fr + T * r * 2 + 2 * out * r * 4 and mr >= inp * r * 2
    assert fr % 256 == 0 and br % 256 == 0 and mr % 256 == 0
    ini = L.loqt_workspace_bytes(L.OP_INIT, 0, out, inp, r)
    assert ini >= out * r * 2 + out * inp * 2 + 2 * r * inp * 4 and ini % 256 == 0
    assert fwd % 256 == 0 and bwd % 256 == 0 and mrg % 256 == 0
    assert L.loqt_workspace_bytes(L.OP_FWD, 0, out, inp, r) == 0
    assert L.loqt_workspace_bytes(L.OP_FWD_NQ, T, out, inp, r) >= T * r * 2
    assert L.loqt_workspace_bytes(L.OP_BWD_NQ, T, out, inp, r) >= T * r * 2 + 2 * r * inp * 4
    assert L.loqt_workspace_bytes(99, T, out, inp, r) == 0
    # the saved pair keeps the weight in the caller's buffer: no out x in copy in the workspace
    assert L.loqt_workspace_bytes(L.OP_FWD_SAVE, T, out, inp, r) <= fwd - out * inp * 2
    assert L.loqt_workspace_bytes(L.OP_BWD_SAVED, T, out, inp, r) <= bwd - out * inp * 2
    assert L.loqt_workspace_bytes(L.OP_BWD_SAVED, T, out, inp, r) >= T * r * 2 + out * r * 2 + r * inp * 4


def test_bad_arguments_are_rejected_before_launch(lib):
    """Every call below must fail in the host-side checks (fake but aligned 'device' addresses
    are never dereferenced there), so this runs without a GPU."""
    from paper_2405_16528_amd import binding as L
    P = 0x10000  # aligned, never touched
    st = lib.nf4_quantize(None, 4, 64, 64, P, P, 64, None)
    assert st == 1
    assert lib.nf4_quantize(P, 4, 64, 64, P, P, 96, None) == 2      # ld_q not a multiple of 64
    assert lib.nf4_quantize(P, 4, 100, 64, P, P, 128, None) == 2     # ld_w < cols
    assert lib.nf4_quantize(P, 0, 64, 64, P, P, 64, None) == 2       # empty
    assert lib.nf4_quantize(P + 4, 4, 64, 64, P, P, 64, None) == 3   # misaligned w
    assert lib.nf4_quantize(P, -1, 64, 64, P, P, 64, None) == 1
    assert lib.nf4_dequantize(P, P, 4, 64, 64, P, 5, 64, None) == 1  # unknown dtype
    assert lib.nf4_dequantize(P, P, 4, 64, 64, P, L.BF16, 36, None) == 2  # bf16 pitch not multiple of 8

    W = L.NF4MatC(P, P, 512, 512, 512)
    Pm = L.NF4MatC(P, P, 512, 128, 128)
    Pbad = L.NF4MatC(P, P, 256, 128, 128)  # rows differ from W
    ws = 1 << 30
    ok_args = dict(x=P, ld_x=512, T=256)
    assert lib.loqt_linear_fwd(P, 512, 256, C.byref(W), C.byref(Pbad), P, 512, 1.0, P, 512, P, ws, None) == 2
    assert lib.loqt_linear_fwd(P, 512, 256, C.byref(W), C.byref(Pm), P, 516, 1.0, P, 512, P, ws, None) == 2
    assert lib.loqt_linear_fwd(P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, None, ws, None) == 1
    assert lib.loqt_linear_fwd(P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P, 16, None) == 4
    assert lib.loqt_linear_fwd(P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P + 16, ws, None) == 3
    assert lib.loqt_linear_fwd(P, 512, 256, None, C.byref(Pm), P, 512, 1.0, P, 512, P, ws, None) == 1
    assert lib.loqt_linear_bwd(P, 512, P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, None, 0, 512, 0,
                               P, ws, None) == 1                                       # dB missing
    assert lib.loqt_linear_bwd(P, 512, P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P, 3, 512, 0,
                               P, ws, None) == 1                                       # unknown dB dtype
    assert lib.loqt_linear_bwd(P, 512, P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P, 0, 100, 0,
                               P, ws, None) == 2                                       # ld_dB < in
    # the pair that keeps the transient 16-bit weight between forward and backward
    fs, bs = lib.loqt_linear_fwd_save, lib.loqt_linear_bwd_saved
    assert fs(P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, None, 512, P, ws, None) == 1   # no w_eff
    assert fs(P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P, 508, P, ws, None) == 2      # pitch < in
    assert fs(P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P + 8, 512, P, ws, None) == 3  # misaligned
    assert fs(P, 512, 256, C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P, 512, P, 16, None) == 4
    assert bs(P, 512, P, 512, 256, C.byref(Pm), 512, 1.0, None, 512, P, 512, P, 0, 512, 0, P, ws, None) == 1
    assert bs(P, 512, P, 512, 256, None, 512, 1.0, P, 512, P, 512, P, 0, 512, 0, P, ws, None) == 1      # no P_q
    assert bs(P, 512, P, 512, 256, C.byref(Pm), -4, 1.0, P, 512, P, 512, P, 0, 512, 0, P, ws, None) == 1
    assert bs(P, 512, P, 512, 256, C.byref(Pm), 512, 1.0, P, 500, P, 512, P, 0, 512, 0, P, ws, None) == 2  # pitch < in
    assert bs(P, 512, P, 512, 256, C.byref(Pm), 512, 1.0, P, 512, P, 512, None, 0, 512, 0, P, ws, None) == 1  # no dB
    assert bs(P, 512, P, 512, 256, C.byref(Pm), 512, 1.0, P, 512, P, 512, P, 0, 512, 0, P, 16, None) == 4
    assert lib.loqt_merge_requant(C.byref(W), None, P, C.byref(Pm), P, 512, 1.0, P, ws, None) == 1
    assert lib.loqt_merge_requant(C.byref(W), P + 64, P, C.byref(Pm), P, 512, 1.0, P, ws, None) == 1  # partial overlap
    assert lib.loqt_merge_requant_batched(-1, None, P, ws, None) == 1
    assert lib.loqt_merge_requant_batched(0, None, P, ws, None) == 0                   # nothing to do
    assert lib.loqt_set_path(9) == 1
    assert lib.loqt_set_path(L.PATH_AUTO) == 0
    assert lib.loqt_set_tile(4) == 1 and lib.loqt_set_tile(-1) == 1
    assert lib.loqt_set_tile(L.TILE_AUTO) == 0

    Qm = L.NF4MatC(P, P, 512, 128, 128)   # in x r
    Qbad = L.NF4MatC(P, P, 256, 128, 128)  # rows differ from W's columns
    assert lib.loqt_linear_fwd_right(P, 512, 256, C.byref(W), C.byref(Qbad), P, 128, 1.0, P, 512, P, ws, None) == 2
    assert lib.loqt_linear_fwd_right(P, 512, 256, C.byref(W), C.byref(Qm), P, 100, 1.0, P, 512, P, ws, None) == 2
    assert lib.loqt_linear_fwd_right(P, 512, 256, C.byref(W), C.byref(Qm), P, 128, 1.0, P, 512, P, 16, None) == 4
    assert lib.loqt_linear_fwd_right(P, 512, 256, C.byref(W), None, P, 128, 1.0, P, 512, P, ws, None) == 1
    assert lib.loqt_linear_bwd_right(P, 512, P, 512, 256, C.byref(W), C.byref(Qm), P, 128, 1.0, P, 512, None, 0, 128,
                                     0, P, ws, None) == 1                              # dBp missing
    assert lib.loqt_linear_bwd_right(P, 512, P, 512, 256, C.byref(W), C.byref(Qm), P, 128, 1.0, P, 512, P, 0, 100,
                                     0, P, ws, None) == 2                              # ld_dBp < r
    assert lib.loqt_merge_requant_right(C.byref(W), None, P, C.byref(Qm), P, 128, 1.0, P, ws, None) == 1
    assert lib.loqt_merge_requant_right(C.byref(W), P + 64, P, C.byref(Qm), P, 128, 1.0, P, ws, None) == 1
    assert lib.loqt_merge_requant_right(C.byref(W), P, P, C.byref(Qm), P, 128, 1.0, None, ws, None) == 1

    assert lib.loqt_merge_dense(C.byref(W), C.byref(Pm), P, 512, 1.0, None, 512, P, ws, None) == 1
    assert lib.loqt_merge_dense(C.byref(W), C.byref(Pm), P, 512, 1.0, P, 510, P, ws, None) == 2
    assert lib.loqt_merge_dense(C.byref(W), C.byref(Pm), P, 512, 1.0, P, 512, P, 16, None) == 4
    assert lib.loqt_adam_step(P, 512, 128, 512, P, 0, 512, P, P, 512, 1e-3, 0.9, 0.999, 1e-8, 0, None) == 1   # step 0
    assert lib.loqt_adam_step(P, 512, 128, 512, P, 0, 512, P, P, 512, 1e-3, 1.0, 0.999, 1e-8, 1, None) == 1   # beta1 = 1
    assert lib.loqt_adam_step(P, 512, 128, 512, P, 7, 512, P, P, 512, 1e-3, 0.9, 0.999, 1e-8, 1, None) == 1   # dtype
    assert lib.loqt_adam_step(P, 512, 128, 512, P, 0, 100, P, P, 512, 1e-3, 0.9, 0.999, 1e-8, 1, None) == 2   # ld_grad
    assert lib.loqt_adam_step(P, 512, 128, 512, None, 0, 512, P, P, 512, 1e-3, 0.9, 0.999, 1e-8, 1, None) == 1
    dqc, dqe = lib.loqt_absmax_dq_compress, lib.loqt_absmax_dq_expand
    dqc.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    dqe.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.loqt_absmax_dq_workspace_bytes.restype = C.c_size_t
    lib.loqt_absmax_dq_workspace_bytes.argtypes = [C.c_int64]
    assert lib.loqt_absmax_dq_workspace_bytes(0) == 0 and lib.loqt_absmax_dq_workspace_bytes(4096 * 64) >= 64 * 8
    assert dqc(None, 1000, P, P, P, P, ws, None) == 1
    assert dqc(P, 0, P, P, P, P, ws, None) == 2
    assert dqc(P + 2, 1000, P, P, P, P, ws, None) == 3
    assert dqc(P, 1000, P, P, P, P, 0, None) == 4
    assert dqe(P, P, None, 1000, P, None) == 1
    assert dqe(P, P, P, -5, P, None) == 2
    assert dqe(P, P + 1, P, 1000, P, None) == 3
    assert lib.loqt_merge_schedule(100.0, 1.2, 2500, 4, None) == 1
    assert lib.loqt_merge_schedule(100.0, 0.5, 2500, 0, (C.c_int64 * 1)()) == 1                            # psi < 1

    assert lib.loqt_linear_fwd_nq(P, 512, 256, None, 512, P, 128, P, 512, 512, 512, 128, 1.0, P, 512, P, ws, None) == 1
    assert lib.loqt_linear_fwd_nq(P, 512, 256, P, 500, P, 128, P, 512, 512, 512, 128, 1.0, P, 512, P, ws, None) == 2
    assert lib.loqt_linear_fwd_nq(P, 512, 256, P, 512, P, 128, P, 512, 512, 512, 128, 1.0, P, 512, P, 16, None) == 4
    assert lib.loqt_linear_bwd_nq(P, 512, P, 512, 256, P, 512, P, 128, P, 512, 512, 512, 128, 1.0, P, 512, None, 0,
                                  512, 0, P, ws, None) == 1
    assert lib.loqt_merge_nq(None, 512, P, 128, P, 512, 512, 512, 128, 1.0, None) == 1
    assert lib.loqt_merge_nq(P, 512, P, 100, P, 512, 512, 512, 128, 1.0, None) == 2

    def init(W=P, ld_w=512, Pp=P, ld_p=128, out=512, inp=512, r=128, s=1.0, iters=3, warm=0, codes=P, am=P, ld_q=512,
             B=P, ld_B=512, w=P, wsb=ws):
        return lib.loqt_init_compensate(W, ld_w, Pp, ld_p, out, inp, r, s, iters, warm, codes, am, ld_q, B, ld_B, w,
                                        wsb, None)
    assert init(W=None) == 1 and init(Pp=None) == 1 and init(codes=None) == 1 and init(B=None) == 1
    assert init(iters=0) == 1 and init(warm=2) == 1 and init(s=0.0) == 1 and init(s=float("nan")) == 1
    assert init(ld_w=510) == 2 and init(ld_p=126) == 2 and init(ld_q=500) == 2 and init(r=0) == 2
    assert init(ld_B=100) == 2
    assert init(W=P + 4) == 3 and init(w=P + 64) == 3
    assert init(w=None) == 1 and init(wsb=1024) == 4


def test_merge_schedule_matches_the_oracle(lib):
    """loqt_merge_schedule is host code: it runs without a GPU and must reproduce the oracle's steps."""
    from oracle import loqt_oracle as O
    from paper_2405_16528_amd import binding as L
    assert L.loqt_merge_schedule(60) == O.merge_schedule(100, 1.2, 2500, 60)
    assert L.loqt_merge_schedule(5, tau=200.0, psi=1.0) == [201, 402, 603, 804, 1005]
    assert L.loqt_merge_schedule(200, tau=50.0, psi=1.5, cap=300) == O.merge_schedule(50, 1.5, 300, 200)
    assert L.loqt_merge_schedule(0) == []


def test_product_plan_is_valid_and_never_worse_than_one_launch(lib):
    """loqt_plan_product is host code.  Whatever the sizes: the 256x256 part is a whole number of tile columns
    short of N, its tiles nearly fill whole rounds of 256, and the plan is never priced above the single launch."""
    from paper_2405_16528_amd import binding as L

    def cdiv(a, b):
        return -(-a // b)

    # the shapes the workloads produce (T, columns, extra columns)
    assert L.plan_product(8192, 4096) == (0, 2.0)                  # two exact rounds
    assert L.plan_product(8192, 11008)[0] == 10240                 # 5.4 rounds: 5 + a 128x128 tail
    assert L.plan_product(8192, 11008, 1024) == (0, 6.0)           # Z rides along and fills the sixth round
    assert L.plan_product(4096, 5120, 1024)[0] == 4096             # 1.25 rounds: 1 + tail that takes Z along
    assert L.plan_product(4096, 5120)[0] == 4096
    for M in (256, 1000, 4096, 8192, 12000):
        for N in (256, 2048, 4096, 5120, 5461, 11008, 13824):
            for Nx in (0, 512, 1024):
                n1, cost = L.plan_product(M, N, Nx)
                one = cdiv(cdiv(M, 256) * (cdiv(N, 256) + cdiv(Nx, 256)), 256)
                assert cost <= one
                if n1:
                    assert n1 % 256 == 0 and 0 < n1 < N
                    tiles_a = cdiv(M, 256) * (n1 // 256)
                    assert tiles_a <= (tiles_a // 256 + 1) * 256 and 256 * cdiv(tiles_a, 256) - tiles_a < 32
                    assert cost < one
                else:
                    assert cost == one
    assert lib.loqt_plan_product(0, 4096, 0, None, None) == 2
    assert lib.loqt_plan_product(4096, 4096, -1, None, None) == 2
    assert lib.loqt_plan_product(4096, 4096, 0, None, None) == 0


def test_static_entry_point_checks_before_any_gpu_call(lib):
    """loqt_absmax_dq_compress_static refuses, on the host, a size beyond its fixed scratch (and the usual misuse)."""
    P = 0x10000
    limit = lib.loqt_absmax_dq_static_max_n()
    assert limit == 1 << 25
    assert lib.loqt_absmax_dq_compress_static(P, limit + 1, P, P, P, None) == 6
    assert lib.loqt_status_string(6) == b"LOQT_STATIC_SCRATCH_TOO_SMALL"
    assert lib.loqt_absmax_dq_compress_static(P, 0, P, P, P, None) == 2
    assert lib.loqt_absmax_dq_compress_static(None, 16, P, P, P, None) == 1
    assert lib.loqt_absmax_dq_compress_static(P + 2, 16, P, P, P, None) == 3


def test_auto_rule_on_the_paper_workloads(lib):
    """Which implementation the default picks (host-side decision, no GPU): the rank-r term is folded into the
    transient weight from T (in + out) >= out in tokens on; the backward pass keeps it as a second K segment of the
    dx product when the weight has more than 0.73 T rows (sec. 2.2: both are the same quantities)."""
    from paper_2405_16528_amd import binding as L
    r = lambda op, T, out, inp: int(lib.loqt_resolved_path(op, T, out, inp))
    # 7B block at 8192 tokens (appendix table of model sizes): q/k/v/o and down fold in both passes, gate / up only forward
    for out, inp in [(4096, 4096), (4096, 11008)]:
        assert r(L.OP_FWD, 8192, out, inp) == L.PATH_FOLDED and r(L.OP_BWD, 8192, out, inp) == L.PATH_FOLDED
    assert r(L.OP_FWD, 8192, 11008, 4096) == L.PATH_FOLDED and r(L.OP_BWD, 8192, 11008, 4096) == L.PATH_PREPASS
    # 13B block at 4096 tokens: every projection has more than 0.73 * 4096 rows
    for out, inp in [(5120, 5120), (13824, 5120), (5120, 13824)]:
        assert r(L.OP_FWD, 4096, out, inp) == L.PATH_FOLDED and r(L.OP_BWD, 4096, out, inp) == L.PATH_PREPASS
    # few tokens: carrying the rank-r term through the tokens is cheaper than folding it
    assert r(L.OP_FWD, 256, 4096, 4096) == L.PATH_PREPASS and r(L.OP_BWD, 256, 4096, 4096) == L.PATH_PREPASS
    # the boundary T (in + out) = out in
    assert r(L.OP_FWD, 2048, 4096, 4096) == L.PATH_FOLDED and r(L.OP_FWD, 2047, 4096, 4096) == L.PATH_PREPASS
