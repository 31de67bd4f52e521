"""The large-tile kernels on small ragged shapes.  The tile shape is normally chosen from the sizes, so the
256x256 and 256x128 tiles (the ones the full-size products run on) only ever see the big workloads; forcing
them here puts their edge handling -- rows, columns and contractions that end inside a tile, contractions
shorter than one k-tile, both storage orders of the B operand -- under the element-by-element comparison
with the oracle."""
import numpy as np
import pytest
import torch

from oracle import loqt_oracle as O
from tests.test_gpu_layer import TOL, _setup, _merge_policy_check

pytestmark = pytest.mark.gpu

SHAPES = [
    # T, out, in, r
    (300, 520, 456, 128),    # ragged in every dimension, K tails of 8
    (515, 1100, 333, 192),   # odd in, K tail 13
    (70, 130, 40, 32),       # everything smaller than one tile
    (777, 264, 1000, 72),    # three row tiles, the last almost empty
    # every contraction a whole number of k-tiles: the kernel variants whose loads carry no mask
    (777, 1088, 1024, 128),
    (128, 128, 64, 64),      # contractions of one and two k-tiles
]


@pytest.fixture(params=["256x256", "256x128"])
def tile(request):
    from paper_2405_16528_amd import binding as L
    L.set_tile({"256x256": L.TILE_256x256, "256x128": L.TILE_256x128}[request.param])
    yield request.param
    L.set_tile(L.TILE_AUTO)


@pytest.fixture(params=["prepass", "folded"])
def path(request):
    from paper_2405_16528_amd import binding as L
    L.set_path({"prepass": L.PATH_PREPASS, "folded": L.PATH_FOLDED}[request.param])
    yield request.param
    L.set_path(L.PATH_AUTO)


@pytest.mark.parametrize("T,out,inp,r", SHAPES)
def test_forced_tiles_fwd_bwd_merge(tile, path, T, out, inp, r):
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    s = 0.5
    lay, Wq, Pq, d = _setup(T, out, inp, r, seed=T + inp, sigma_B=2e-2)
    y = G.bf16_empty(T, out, fill=float("nan"))
    dx = G.bf16_empty(T, inp, fill=float("nan"))
    dB = torch.full((r, inp), float("nan"), dtype=torch.float32, device="cuda")
    L.loqt_linear_fwd(d["x"], d["Wq"], d["Pq"], d["B"], s, y, G.workspace(L.OP_FWD, T, out, inp, r))
    L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], s, dx, dB, False,
                      G.workspace(L.OP_BWD, T, out, inp, r))
    # the merge with an update of the size the workloads have (B ~ 1e-3), as in the merge parity test
    lay_m, _, _, dm = _setup(T, out, inp, r, seed=T + inp)
    merged = L.loqt_merge_requant(dm["Wq"], dm["Pq"], dm["B"], s, out=L.NF4Tensor.empty(out, inp))
    torch.cuda.synchronize()
    y_ref = O.loqt_linear_fwd(lay.x, Wq, Pq, lay.B, s)
    dx_ref, dB_ref = O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, s)
    ey = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(y)), y_ref)
    ex = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dx)), dx_ref)
    eb = G.max_err_over_rms(dB.cpu().numpy().astype(np.float64), dB_ref)
    print(f"tile {tile} path {path} T={T} out={out} in={inp} r={r}: err/rms y {ey:.2e} dx {ex:.2e} dB {eb:.2e}")
    assert ey <= TOL and ex <= TOL and eb <= TOL
    c, a, _, _ = G.nf4_host(merged)
    rate = _merge_policy_check(c, a, Wq, Pq, lay_m.B, s)
    assert rate <= 1e-3


def test_forced_tiles_match_auto_bitwise_where_order_is_the_same(tile):
    """The same contraction order per output element (k ascending in steps of 64, fp32 accumulation inside
    the matrix unit) holds for every tile shape with the 32x32x16 instruction, so the merge, whose epilogue
    is the same code, must give identical codes whatever the tile."""
    from paper_2405_16528_amd import binding as L
    T, out, inp, r = 64, 392, 448, 96
    lay, Wq, Pq, d = _setup(T, out, inp, r, seed=5, sigma_B=2e-2)
    L.set_path(L.PATH_PREPASS)
    try:
        forced = L.loqt_merge_requant(d["Wq"], d["Pq"], d["B"], 1.0, out=L.NF4Tensor.empty(out, inp))
        L.set_tile(L.TILE_AUTO)
        auto = L.loqt_merge_requant(d["Wq"], d["Pq"], d["B"], 1.0, out=L.NF4Tensor.empty(out, inp))
        torch.cuda.synchronize()
    finally:
        L.set_path(L.PATH_AUTO)
    assert torch.equal(forced.codes, auto.codes) and torch.equal(forced.absmax, auto.absmax)


@pytest.mark.parametrize("T,out,inp,r", [(300, 520, 456, 128), (130, 1000, 300, 64)])
def test_forced_tiles_right_side(tile, T, out, inp, r):
    """The right-side form (sec. 2.2: projection on the input side) uses other operand orders of the same kernels."""
    from tests import gpu_util as G
    from tests.test_gpu_right import _setup as _setup_right
    from paper_2405_16528_amd import binding as L
    s = 0.5
    Wq, Qq, Bp, x, dy, d = _setup_right(T, out, inp, r, seed=T + out)
    y = G.bf16_empty(T, out, fill=float("nan"))
    dx = G.bf16_empty(T, inp, fill=float("nan"))
    dBp = torch.full((out, r), float("nan"), dtype=torch.float32, device="cuda")
    L.loqt_linear_fwd_right(d["x"], d["Wq"], d["Qq"], d["Bp"], s, y, G.workspace(L.OP_FWD_RIGHT, T, out, inp, r))
    L.loqt_linear_bwd_right(d["dy"], d["x"], d["Wq"], d["Qq"], d["Bp"], s, dx, dBp, False,
                            G.workspace(L.OP_BWD_RIGHT, T, out, inp, r))
    torch.cuda.synchronize()
    y_ref = O.loqt_linear_fwd_right(x, Wq, Qq, Bp, s)
    dx_ref, dB_ref = O.loqt_linear_bwd_right(dy, x, Wq, Qq, Bp, s)
    ey = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(y)), y_ref)
    ex = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dx)), dx_ref)
    eb = G.max_err_over_rms(dBp.cpu().numpy().astype(np.float64), dB_ref)
    print(f"tile {tile} right T={T} out={out} in={inp} r={r}: err/rms y {ey:.2e} dx {ex:.2e} dBp {eb:.2e}")
    assert ey <= TOL and ex <= TOL and eb <= TOL


@pytest.mark.parametrize("T", [70, 128, 200, 1024, 1100])
def test_rank_1024_gradient_on_the_wide_tiles(T):
    """From rank 1024 up the fp32 slices of dB run on 256x128 tiles (16x16x32 loop, masked-load variant when the
    contraction does not end on a k-tile), whatever the other sizes: contractions (over T) of two k-tiles with a
    short last one, of exactly two, of four with a short last one, of sixteen whole ones, and of two slices with a
    short last k-tile."""
    from tests import gpu_util as G
    from paper_2405_16528_amd import binding as L
    out, inp, r, s = 1100, 200, 1024, 0.5
    L.set_path(L.PATH_FOLDED)
    try:
        lay, Wq, Pq, d = _setup(T, out, inp, r, seed=T, sigma_B=2e-2)
        dx = G.bf16_empty(T, inp, fill=float("nan"))
        dB = torch.full((r, inp), float("nan"), dtype=torch.float32, device="cuda")
        L.loqt_linear_bwd(d["dy"], d["x"], d["Wq"], d["Pq"], d["B"], s, dx, dB, False,
                          G.workspace(L.OP_BWD, T, out, inp, r))
        torch.cuda.synchronize()
    finally:
        L.set_path(L.PATH_AUTO)
    dx_ref, dB_ref = O.loqt_linear_bwd(lay.dy, lay.x, Wq, Pq, lay.B, s)
    ex = G.max_err_over_rms(O.bf16_to_f64(G.bf16_host(dx)), dx_ref)
    eb = G.max_err_over_rms(dB.cpu().numpy().astype(np.float64), dB_ref)
    print(f"r=1024 T={T}: err/rms dx {ex:.2e} dB {eb:.2e}")
    assert ex <= TOL and eb <= TOL
