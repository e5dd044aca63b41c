"""GPU parity: libtoma (through the C ABI) against the fp64 CPU oracle, element by element on the
same seeded inputs.  Destination indices must be identical (near ties: see toma_gpu.compare_picks);
floating-point outputs within max|err| / max|ref| <= 1e-4 (fp32) or 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

from paper_2509_10918_amd import binding as tb
from paper_2509_10918_amd import synth

import toma_gpu as tg

pytestmark = pytest.mark.gpu

W = synth.WORKLOADS
SMALL_BF16 = synth.scaled(W["sdxl1"], name="small_bf16", B=2, H=32, W=48, C=96, tile_h=16, tile_w=16, heads=3,
                          sigma=1.5)
RAGGED_F32 = synth.scaled(W["tiny"], name="ragged_f32", B=2, H=24, W=16, C=64, tile_h=12, tile_w=4, keep=0.4375,
                          heads=2, index=7)
STRIPE_BF16 = synth.scaled(W["sdxl1"], name="stripe", B=1, H=16, W=32, C=64, tile_h=2, tile_w=32, keep=0.25,
                           heads=1, index=8)
EXTRA_BF16 = synth.scaled(W["flux"], name="extra", B=1, H=32, W=32, C=256, tile_h=16, tile_w=16, heads=2,
                          T_extra=72, index=9)
CASES = {"tiny": W["tiny"], "small_bf16": SMALL_BF16, "ragged_f32": RAGGED_F32, "stripe": STRIPE_BF16,
         "extra": EXTRA_BF16}


def _f64(a):
    return np.asarray(a, dtype=np.float64)


@pytest.fixture(scope="module")
def cases():
    return {k: (w, synth.make_inputs(w)) for k, w in CASES.items()}


@pytest.mark.parametrize("name", list(CASES))
def test_select_matches_oracle_exactly(oracle, cases, name):
    w, inp = cases[name]
    print(f"[select] {name} B={w.B} N={w.N} C={w.C} n_loc={w.n_loc} d_loc={w.d_loc}", flush=True)
    dv = tg.Device(w, inp, 1)
    idx = dv.select()
    bad, near, forced = tg.compare_picks(oracle, w, _f64(inp["X"]), idx)
    print(f"  near-tie steps {near}, regions verified teacher-forced {forced}, mismatching {bad}", flush=True)
    assert not bad
    # reported gains are the oracle's winning values
    d = tg.oracle_desc(oracle, w, 1)
    idx_ref, gain_ref, gap_ref = oracle.select(d, _f64(inp["X"]))
    same = np.all(idx == idx_ref, axis=2)
    got = dv.gain.cpu().numpy()
    assert np.allclose(got[same], gain_ref[same], rtol=1e-6, atol=1e-6)
    # reported leads over the runner-up are the oracle's: both sides hold them exactly on the grid, so
    # exact ties are zeros on both sides and the near-tie report (gap / gain < 1e-6) is the same set
    gap = dv.gap.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isinf(gap[same]), np.isinf(gap_ref[same]))
    fin = same[..., None] & np.isfinite(gap_ref)
    assert np.allclose(gap[fin], gap_ref[fin], rtol=1e-6, atol=0.0)
    assert np.array_equal(gap[fin] == 0.0, gap_ref[fin] == 0.0)
    near_gpu = gap[fin] < tg.NEAR_TIE * np.maximum(got.astype(np.float64)[fin], 1e-30)
    near_ref = gap_ref[fin] < tg.NEAR_TIE * np.maximum(gain_ref[fin], 1e-30)
    # (float32 rounding of the reported pair could move a gap sitting exactly on the threshold)
    assert int((near_gpu != near_ref).sum()) <= 1
    print(f"  near ties reported by the library: {int(near_gpu.sum())}, by the oracle: {int(near_ref.sum())}", flush=True)
    # the picks do not depend on whether the lead is asked for
    assert np.array_equal(dv.select(gap=False), idx)


@pytest.mark.parametrize("n_loc_shape,d_loc", [((4, 4), 16), ((4, 4), 1), ((8, 6), 7), ((16, 16), 256),
                                               ((10, 16), 33), ((16, 13), 100)])
def test_select_region_sizes(oracle, n_loc_shape, d_loc):
    th, tw = n_loc_shape
    w = synth.scaled(W["tiny"], name="sel", B=2, H=2 * th, W=3 * tw, C=32, tile_h=th, tile_w=tw,
                     keep=d_loc / (th * tw), index=11)
    assert w.d_loc == d_loc
    print(f"[select sizes] tile {th}x{tw} d_loc={d_loc}", flush=True)
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    bad, near, forced = tg.compare_picks(oracle, w, _f64(inp["X"]), dv.select())
    assert not bad


@pytest.mark.parametrize("dtype,grid,tile,keep", [
    ("f32", (32, 32), (32, 32), 0.25),      # one region of 1024 tokens per sample: the paper's few-regions end
    ("bf16", (64, 32), (32, 32), 0.5),      # two regions of 1024
    ("bf16", (24, 48), (24, 24), 0.125),    # 576 tokens: not a multiple of the workgroup's 1024 threads
    ("f32", (32, 64), (32, 64), 0.0625),    # 2048 tokens: two rows and two columns per thread
])
def test_select_large_regions(oracle, dtype, grid, tile, keep):
    """Regions of more than 256 tokens take the selection kernel that keeps the similarities in memory:
    picks, reported gains and leads over the runner-up must be the oracle's, exactly."""
    H, Wd = grid
    th, tw = tile
    w = synth.scaled(W["tiny"], name="bigregion", dtype=dtype, B=2, H=H, W=Wd, C=64, tile_h=th, tile_w=tw, keep=keep,
                     heads=1, index=23)
    print(f"[select large regions] {dtype} grid {H}x{Wd} tile {th}x{tw} n_loc={w.n_loc} d_loc={w.d_loc}", flush=True)
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    idx = dv.select()
    bad, near, forced = tg.compare_picks(oracle, w, _f64(inp["X"]), idx)
    print(f"  near-tie steps {near}, regions verified teacher-forced {forced}, mismatching {bad}", flush=True)
    assert not bad
    d = tg.oracle_desc(oracle, w, 1)
    idx_ref, gain_ref, gap_ref = oracle.select(d, _f64(inp["X"]))
    assert np.array_equal(idx, idx_ref)
    assert np.allclose(dv.gain.cpu().numpy(), gain_ref, rtol=1e-6, atol=1e-6)
    gap = dv.gap.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isinf(gap), np.isinf(gap_ref))
    fin = np.isfinite(gap_ref)
    assert np.allclose(gap[fin], gap_ref[fin], rtol=1e-6, atol=0.0)
    assert np.array_equal(gap[fin] == 0.0, gap_ref[fin] == 0.0)
    assert np.array_equal(dv.select(gap=False), idx)


@pytest.mark.parametrize("dtype,tile,keep", [
    ("bf16", (4, 4), 0.5),       # 16 tokens: one wave, one row per lane
    ("f32", (8, 16), 0.5),       # 128 tokens: four waves, two rows per lane, rotated column ownership
    ("bf16", (16, 8), 0.25),     # 128 tokens in a narrow tile
    ("f32", (10, 16), 0.3),      # 160 tokens: five waves (the tile width is no multiple: plain ownership)
    ("bf16", (16, 12), 0.25),    # 192 tokens, a tile width that is no power of two
    ("bf16", (13, 16), 0.5),     # 208 tokens: four rows per lane with lanes and registers past the end
    ("f32", (15, 16), 0.5),      # 240 tokens: eight waves, 30 of 32 registers per wave in use
    ("bf16", (8, 32), 0.75),     # 256 tokens in a wide tile, three quarters kept
])
def test_select_region_sizes(oracle, dtype, tile, keep):
    """Region sizes between the smallest and 256 tokens: every number of waves and rows per lane of the
    register-resident selection kernel, with and without the rotated assignment of columns to waves,
    and regions that leave lanes, registers and LDS slots past their end unused.  Picks, gains and leads
    must be the oracle's."""
    th, tw = tile
    w = synth.scaled(W["tiny"], name="regionsize", dtype=dtype, B=2, H=2 * th, W=tw, C=64, tile_h=th, tile_w=tw,
                     keep=keep, heads=1, index=29)
    print(f"[select region sizes] {dtype} tile {th}x{tw} n_loc={w.n_loc} d_loc={w.d_loc}", flush=True)
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    idx = dv.select()
    bad, near, forced = tg.compare_picks(oracle, w, _f64(inp["X"]), idx)
    print(f"  near-tie steps {near}, regions verified teacher-forced {forced}, mismatching {bad}", flush=True)
    assert not bad
    d = tg.oracle_desc(oracle, w, 1)
    idx_ref, gain_ref, gap_ref = oracle.select(d, _f64(inp["X"]))
    same = np.all(idx == idx_ref, axis=2)
    assert same.any()
    assert np.allclose(dv.gain.cpu().numpy()[same], gain_ref[same], rtol=1e-6, atol=1e-6)
    gap = dv.gap.cpu().numpy().astype(np.float64)
    fin = same[..., None] & np.isfinite(gap_ref)
    assert np.allclose(gap[fin], gap_ref[fin], rtol=1e-6, atol=0.0)
    assert np.array_equal(dv.select(gap=False), idx)


def test_select_on_random_shapes(oracle):
    """A seeded sweep over grids, tile shapes, channel counts, keep ratios and both dtypes (regions of 16
    to 256 tokens, several regions along both axes, three samples): picks must be the oracle's."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 14:
        th, tw = int(rng.integers(1, 17)), int(rng.choice([2, 4, 8, 12, 16, 24, 32, 64]))
        n_loc = th * tw
        if n_loc % 16 or n_loc > 256:
            continue
        gh, gw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        d_loc = int(rng.integers(1, n_loc + 1))
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        C = int(rng.choice([32, 64, 96, 160]))
        w = synth.scaled(W["tiny"], name="rand", dtype=dtype, B=3, H=gh * th, W=gw * tw, C=C, tile_h=th, tile_w=tw,
                         keep=d_loc / n_loc, heads=1, index=100 + done)
        if w.d_loc != d_loc:
            continue
        print(f"[select random shapes] {dtype} grid {gh}x{gw} tiles of {th}x{tw}, C={C}, d_loc={d_loc}", flush=True)
        inp = synth.make_inputs(w)
        desc = tb.make_desc(w.B, w.H, w.W, w.C, w.tile_h, w.tile_w, w.d_loc, 1, w.tau, w.dtype)
        X = tg.dev(inp["X"], dtype)
        ws = tb.alloc_workspace(desc)
        idx = torch.empty((w.B, w.P, w.d_loc), dtype=torch.int32, device="cuda")
        tb.toma_select(desc, X, idx, None, None, ws)
        torch.cuda.synchronize()
        bad, near, forced = tg.compare_picks(oracle, w, _f64(inp["X"]), idx.cpu().numpy())
        assert not bad, (th, tw, gh, gw, d_loc, dtype, C)
        done += 1


def test_layer_with_large_regions(oracle):
    """A whole layer call whose selection regions hold 1024 tokens (global merge), against the oracle."""
    w = synth.scaled(W["tiny"], name="biglayer", dtype="bf16", B=2, H=32, W=64, C=128, tile_h=32, tile_w=32, keep=0.25,
                     heads=2, index=29)
    inp = synth.make_inputs(w)
    X = _f64(inp["X"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    ref = oracle.layer(tg.oracle_desc(oracle, w, 1), X, *Wts, heads=w.heads)
    dv = tg.Device(w, inp, 1)
    Y, _ = dv.layer(0)
    assert np.array_equal(dv.idx.cpu().numpy(), ref["idx"])
    _check_stage("Y", Y, ref["Y"], tg.TOL[w.dtype])


@pytest.mark.parametrize("dtype,C", [("bf16", 128), ("bf16", 256), ("f32", 64)])
def test_select_many_regions(oracle, dtype, C):
    """64 regions of 256 tokens: enough 32 x 32 blocks of the similarity matrices for the kernel that
    takes them whole, with K in one slice (few channels) and in two; the picks must be the oracle's."""
    w = synth.scaled(W["tiny"], name="many", dtype=dtype, B=1, H=128, W=128, C=C, tile_h=16, tile_w=16,
                     keep=0.25, heads=max(1, C // 64), index=17)
    print(f"[select many regions] {dtype} C={C} regions={w.P}", flush=True)
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    bad, near, forced = tg.compare_picks(oracle, w, _f64(inp["X"]), dv.select())
    assert not bad


def test_select_all_identical_tokens_picks_in_index_order(oracle):
    w = synth.scaled(W["tiny"], name="const", B=1, H=8, W=8, C=32, tile_h=4, tile_w=4, keep=1.0, index=12)
    inp = synth.make_inputs(w)
    inp["X"] = np.ones_like(inp["X"])
    dv = tg.Device(w, inp, 1)
    idx = dv.select()
    _, _, token_of = oracle.region_map(8, 8, 4, 4)
    assert np.array_equal(idx[0], token_of)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_select_with_zero_tokens(oracle, dtype):
    """Tokens that are all zeros have no direction: their norm is clamped at 1e-12, every similarity
    with them is 0 (also with themselves), and they compete like any other token.  A zero token, a
    pair of them in one region and a region that is half zeros, against the oracle's picks."""
    w = synth.scaled(W["sdxl1"], name="zeros", dtype=dtype, B=1, H=32, W=32, C=64, tile_h=16, tile_w=16, heads=1,
                     sigma=1.5, index=19)
    inp = synth.make_inputs(w)
    _, _, token_of = oracle.region_map(w.H, w.W, w.tile_h, w.tile_w)
    X = inp["X"].copy()
    X[0, token_of[0][37]] = 0.0
    X[0, token_of[1][[3, 200]]] = 0.0
    X[0, token_of[2][::2]] = 0.0
    inp["X"] = X
    dv = tg.Device(w, inp, 1)
    idx = dv.select()
    bad, near, forced = tg.compare_picks(oracle, w, _f64(X), idx)
    print(f"[select zeros] {dtype}: near-tie steps {near}, teacher-forced {forced}, mismatching {bad}", flush=True)
    assert not bad
    d = tg.oracle_desc(oracle, w, 1)
    idx_ref, gain_ref, _ = oracle.select(d, _f64(X))
    assert np.array_equal(idx, idx_ref)
    assert np.allclose(dv.gain.cpu().numpy(), gain_ref, rtol=1e-6, atol=1e-6)


@pytest.mark.parametrize("C,heads", [(1024, 16), (672, 21)])   # (672: the last 64-channel chunk of a row is half padding)
def test_select_with_elements_far_below_a_tokens_largest(oracle, C, heads):
    """bf16 tokens are compared in fixed point against each token's largest exponent; an element more
    than 22 binary orders below it does not fit: a few such elements per token are added back exactly
    after the fixed-point product, a token with many has its similarities recomputed in double precision.
    Tokens with tiny, subnormal and huge elements next to ordinary ones: the picks and the reported
    values must still be the oracle's, which knows nothing of either path."""
    w = synth.scaled(W["sdxl1"], name="range", B=2, H=64, W=64, C=C, tile_h=16, tile_w=16, heads=heads, sigma=1.5, index=31)
    assert w.B * w.P * 10 * ((w.C + 63) // 64) >= 3000   # enough blocks of S x channel chunks for the fixed-point kernel to run
    inp = synth.make_inputs(w)
    _, _, token_of = oracle.region_map(w.H, w.W, w.tile_h, w.tile_w)
    X = inp["X"].copy()
    X[0, token_of[0][5], 17] = 3e-9          # 29 orders below the token's largest: flagged
    X[0, token_of[0][5], C - 25] = -7e-12
    X[0, token_of[0][6], 17] = 1e-9          # the same channel dropped from two tokens of one region
    X[0, token_of[1][100], 0] = 1e-40        # a bf16 subnormal
    X[1, token_of[2][31], C - 32] = 2.5e4       # a huge element: everything else of the token is far below it
    X[1, token_of[2][32], 3] = -1.0e6        # (bits of the ordinary elements drop out: flagged)
    X[1, token_of[3][7]] *= 1e-6             # a token that is small as a whole: not flagged, same direction
    X[0, token_of[9][200]] = 0.0             # a token without direction
    X[1, token_of[15][255], 1:] = 0.0        # a token with one nonzero element
    X = synth.round_to_bf16(X)
    inp["X"] = X
    dv = tg.Device(w, inp, 1)
    idx = dv.select()
    d = tg.oracle_desc(oracle, w, 1)
    idx_ref, gain_ref, gap_ref = oracle.select(d, _f64(X))
    bad, near, forced = tg.compare_picks(oracle, w, _f64(X), idx)
    print(f"[select range] near-tie steps {near}, teacher-forced {forced}, mismatching {bad}", flush=True)
    assert not bad
    assert np.array_equal(idx, idx_ref)
    assert np.allclose(dv.gain.cpu().numpy(), gain_ref, rtol=1e-6, atol=1e-6)


def _check_stage(name, got, ref, tol):
    err = tg.max_rel(got, ref)
    ex = tg.elem_excess(got, ref, tol)
    print(f"  {name}: max|err|/max|ref| = {err:.3e} (tol {tol:g}); element-wise excess {ex:.3f}", flush=True)
    assert np.all(np.isfinite(got)) and err <= tol, name
    assert ex <= tg.MAX_ELEM_EXCESS, name


@pytest.mark.parametrize("tile_local", [False, True])
@pytest.mark.parametrize("name", list(CASES))
def test_stages_isolated(oracle, cases, name, tile_local):
    """Each stage is fed the oracle's result of the previous one (rounded to the dtype)."""
    w, inp = cases[name]
    R = w.P if tile_local else 1
    tol = tg.TOL[w.dtype]
    print(f"[stages] {name} merge_regions={R}", flush=True)
    X = _f64(inp["X"])
    Xe = None if inp["X_extra"] is None else _f64(inp["X_extra"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, R)
    ref = oracle.layer(d, X, *Wts, heads=w.heads, Xe=Xe)
    print(f"  destinations with Z < 1e-20 (clamped): {ref['clamps']}", flush=True)
    dv = tg.Device(w, inp, R)
    A, Z, Xm = dv.merge(idx=ref["idx"])
    At_ref = ref["A"] / np.maximum(ref["Z"], 1e-20).reshape(w.B, R, -1, 1)
    At = A / np.maximum(Z, 1e-20).reshape(w.B, R, -1, 1)
    _check_stage("A~", At, At_ref, tol)
    _check_stage("Z", Z, ref["Z"], tol)
    _check_stage("Xm", Xm, ref["Xm"], tol)
    # merge with cached weights reproduces the merge bit for bit
    assert np.array_equal(dv.merge_cached(), Xm)
    Xm_in = synth.quantize(w, ref["Xm"])
    O = dv.attend(Xm=Xm_in)
    O_ref = oracle.attend(_f64(Xm_in), Xe, *Wts, heads=w.heads)
    _check_stage("O", O, O_ref, tol)
    O_in = synth.quantize(w, O_ref)
    Y = dv.unmerge(O=O_in)
    Zg = np.maximum(Z, 1e-20)
    Y_ref = oracle.unmerge(d, A, Zg, _f64(O_in))       # the GPU's own stored (A, Z) applied in fp64
    _check_stage("Y (GPU weights)", Y, Y_ref, tol)
    Y_ref2 = oracle.unmerge(d, ref["A"], ref["Z"], _f64(O_in))
    _check_stage("Y (oracle weights)", Y, Y_ref2, tol)


@pytest.mark.parametrize("dtype,grid,tile,keep,C,passes", [
    ("bf16", (16, 16), (8, 8), 0.5, 64, 1),      # 128 destinations: one 128-wide slice per workgroup
    ("f32", (32, 16), (8, 8), 0.5, 32, 1),       # 256 destinations
    ("bf16", (32, 32), (8, 8), 0.5, 128, 1),     # 512 destinations
    ("bf16", (32, 64), (16, 16), 0.5, 64, 1),    # 1024 destinations
    ("f32", (64, 64), (16, 16), 0.5, 32, 1),     # 2048 destinations: the largest single-pass case
    ("bf16", (32, 48), (8, 8), 0.5, 64, 2),      # 768 destinations: not a single-pass size
    ("bf16", (16, 16), (8, 8), 0.25, 64, 2),     # 64 destinations: not a single-pass size
    ("bf16", (32, 64), (16, 16), 0.5, 1024, 2),  # 1024 destinations, 16 K steps, 128 workgroups: two passes are cheaper
])
def test_merge_weights_region_sizes(oracle, dtype, grid, tile, keep, C, passes):
    """Global merge weights over every destination count the single-pass kernel is instantiated for,
    sizes it does not take and a shape where two passes are cheaper, against the oracle's A / Z, Z
    and merged tokens; the profiling aid says which path ran."""
    H, Wd = grid
    th, tw = tile
    w = synth.scaled(W["tiny"], name="wsize", dtype=dtype, B=2, H=H, W=Wd, C=C, tile_h=th, tile_w=tw, keep=keep,
                     heads=max(1, C // 128), index=13)
    print(f"[weights sizes] {dtype} grid {H}x{Wd} tile {th}x{tw} D={w.D} C={C}", flush=True)
    inp = synth.make_inputs(w)
    tol = tg.TOL[dtype]
    X = _f64(inp["X"])
    d = tg.oracle_desc(oracle, w, 1)
    idx, _, _ = oracle.select(d, X)
    A_ref, Z_ref, _ = oracle.merge_weights(d, X, idx)
    Xm_ref = oracle.merge(d, X, A_ref, Z_ref)
    dv = tg.Device(w, inp, 1)
    tb.toma_profile_enable(True)
    try:
        tb.toma_profile_read("weights_stats")
        A, Z, Xm = dv.merge(idx=idx)
        stats_launches, _ = tb.toma_profile_read("weights_stats")
    finally:
        tb.toma_profile_enable(False)
    assert stats_launches == (1 if passes == 2 else 0)
    At_ref = A_ref / np.maximum(Z_ref, 1e-20).reshape(w.B, 1, -1, 1)
    At = A / np.maximum(Z, 1e-20).reshape(w.B, 1, -1, 1)
    _check_stage("A~", At, At_ref, tol)
    _check_stage("Z", Z, Z_ref, tol)
    _check_stage("Xm", Xm, Xm_ref, tol)
    # every source token's weights over the destinations sum to one (softmax over destinations)
    assert np.allclose(A.sum(axis=2), 1.0, atol=3 * tol)


@pytest.mark.parametrize("dtype,tau,C,passes", [("bf16", 0.1, 64, 1), ("bf16", 0.5, 64, 1), ("bf16", 3.0, 64, 1), ("bf16", 100.0, 64, 1),
                                                 ("bf16", 3.0, 1024, 2), ("bf16", 100.0, 1024, 2),
                                                 ("f32", 0.1, 32, 1), ("f32", 2.0, 32, 1)])
def test_merge_unmerge_skip_only_empty_blocks(oracle, dtype, tau, C, passes):
    """The merge and unmerge products walk only the K steps whose blocks of the stored weights hold a
    nonzero value.  Temperatures from almost one-hot weights (most blocks empty) to almost uniform
    ones (no block empty), with the map written by the single-pass weights kernel, by the two-pass
    write and by the scan of a cached A: every result must equal the dense definition."""
    big = C > 64
    w = synth.scaled(W["tiny"], name="occ", dtype=dtype, B=2, H=32 if big else 64, W=64, C=C, tile_h=16, tile_w=16,
                     keep=0.5, heads=max(1, C // 128), tau=tau, index=15)
    print(f"[occupancy] {dtype} tau={tau} C={C} N={w.N} D={w.D}", flush=True)
    inp = synth.make_inputs(w)
    tol = tg.TOL[dtype]
    rng = np.random.default_rng(11)
    X = _f64(inp["X"])
    d = tg.oracle_desc(oracle, w, 1)
    idx, _, _ = oracle.select(d, X)
    A_ref, Z_ref, _ = oracle.merge_weights(d, X, idx)
    Xm_ref = oracle.merge(d, X, A_ref, Z_ref)
    dv = tg.Device(w, inp, 1)
    tb.toma_profile_enable(True)
    try:
        tb.toma_profile_read("weights_stats")
        A, Z, Xm = dv.merge(idx=idx)                       # map from the weights kernels
        stats_launches, _ = tb.toma_profile_read("weights_stats")
    finally:
        tb.toma_profile_enable(False)
    assert stats_launches == (1 if passes == 2 else 0)
    _check_stage("Xm", Xm, Xm_ref, tol)
    nonzero = float((A != 0).mean())
    print(f"  nonzero fraction of the stored weights: {nonzero:.4f}", flush=True)
    if dtype == "bf16":   # (fp32 keeps far smaller weights above zero)
        assert (nonzero < 0.05) if tau <= 0.1 else (nonzero > 0.9 if tau > 50 else True)
    # cached pattern: the oracle's weights (rounded to the dtype) go to the device, the map comes
    # from the scan of that A
    A_in = _f64(synth.quantize(w, A_ref.astype(np.float32)))
    dv.plant(A_in, Z_ref)
    _check_stage("Xm (cached A)", dv.merge_cached(), oracle.merge(d, X, A_in, Z_ref), tol)
    O = synth.quantize(w, rng.standard_normal((w.B, w.D, w.C)).astype(np.float32))
    Y = dv.unmerge(O=O)
    _check_stage("Y", Y, oracle.unmerge(d, A_in, np.maximum(Z_ref, 1e-20), _f64(O)), tol)


def _crafted_weights(rng, B, D, N, case):
    """Sparse weights [B, D, N] with the sources in the order the library stores them: one to three
    destinations per source, all inside the source's own 128-destination block, plus what the case
    plants."""
    A = np.zeros((B, D, N), dtype=np.float32)
    per_block = N // (D // 128)            # sources whose destinations lie in one block
    for b in range(B):
        for i in range(N):
            blk = i // per_block
            for j in rng.choice(128, size=int(rng.integers(1, 4)), replace=False):
                A[b, blk * 128 + j, i] = rng.uniform(0.1, 1.0)
    if case == "long row":                 # 65 weights in one destination's row
        A[1, 300, :] = 0.0
        A[1, 300, rng.choice(N, size=65, replace=False)] = 0.5
    elif case == "many source blocks":     # 65 occupied blocks of 32 sources in one destination block
        A[0, 128:256, :] = 0.0
        for k in range(65):
            A[0, 128 + k, 32 * (k + 3) + 5] = 0.25
    elif case == "many destination blocks":  # a block of 32 sources with weights in 9 destination blocks
        A[0, :, 64:96] = 0.0
        for k in range(9):
            A[0, 128 * k + 7, 64 + k] = 0.75
    elif case == "long column":            # 17 weights for one source, in one destination block
        A[1, :, 1000] = 0.0
        A[1, 512 + 3 * np.arange(17), 1000] = 0.125
    elif case == "crowded rows":           # 16 rows x 32 sources with 80 weights
        A[0, 256:272, 512:544] = 0.0
        for r in range(16):
            A[0, 256 + r, 512 + rng.choice(32, size=5, replace=False)] = 0.375
    elif case == "empty":                  # a destination nobody chooses and a source with no weight at all
        A[0, 40, :] = 0.0
        A[1, :, 77] = 0.0
    return A


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("case", ["plain", "empty", "long row", "many source blocks", "many destination blocks",
                                  "long column", "crowded rows"])
def test_merge_unmerge_of_planted_weights(oracle, dtype, case):
    """Merge and unmerge of a cached, planted A on a shape long enough for the occupancy map: very
    sparse weights around the block diagonal plus rows, columns and blocks that are far denser or
    far more scattered than the rest.  Whatever blocks the products skip, the result is the dense
    definition; then the same through the layer call with the cached pattern."""
    print(f"[planted] {dtype} {case}", flush=True)
    w = synth.scaled(W["tiny"], name="planted", dtype=dtype, B=2, H=64, W=64, C=128, tile_h=16, tile_w=16,
                     keep=0.5, heads=2, index=16)
    inp = synth.make_inputs(w)
    tol = tg.TOL[dtype]
    rng = np.random.default_rng(21)
    d = tg.oracle_desc(oracle, w, 1)
    dv = tg.Device(w, inp, 1)
    A_in = tg.a_in_oracle_order(dv.desc, _f64(synth.quantize(w, _crafted_weights(rng, w.B, w.D, w.N, case))))
    Z = A_in.sum(axis=2)
    X = _f64(inp["X"])
    dv.plant(A_in, Z)
    _check_stage("Xm", dv.merge_cached(), oracle.merge(d, X, A_in, Z), tol)
    O = synth.quantize(w, rng.standard_normal((w.B, w.D, w.C)).astype(np.float32))
    _check_stage("Y", dv.unmerge(O=O), oracle.unmerge(d, A_in, np.maximum(Z, 1e-20), _f64(O)), tol)
    Yl, _ = dv.layer(tb.TOMA_REUSE_A)
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    ref = oracle.layer(d, X, *Wts, heads=w.heads, idx=np.zeros((w.B, w.P, w.d_loc), dtype=np.int64), AZ=(A_in, Z))
    _check_stage("Y (layer, cached A)", Yl, ref["Y"], tol)


@pytest.mark.parametrize("tile_local", [False, True])
@pytest.mark.parametrize("name", list(CASES))
def test_layer_chained_and_reuse(oracle, cases, name, tile_local):
    w, inp = cases[name]
    R = w.P if tile_local else 1
    tol = tg.TOL[w.dtype]
    print(f"[layer] {name} merge_regions={R}", flush=True)
    X = _f64(inp["X"])
    Xe = None if inp["X_extra"] is None else _f64(inp["X_extra"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, R)
    ref = oracle.layer(d, X, *Wts, heads=w.heads, Xe=Xe)
    dv = tg.Device(w, inp, R)
    Y, Ye = dv.layer(0)
    bad, near, forced = tg.compare_picks(oracle, w, X, dv.idx.cpu().numpy())
    assert not bad
    _check_stage("Y", Y, ref["Y"], tol)
    if Ye is not None:
        _check_stage("Y_extra", Ye, ref["Y_extra"], tol)
    # bit-identical rerun (no atomics, fixed reduction orders)
    Y2, _ = dv.layer(0)
    assert np.array_equal(Y, Y2)
    # pattern reuse on drifted tokens: cached idx, then cached (A, Z)
    rng = np.random.default_rng(99)
    X1 = synth.quantize(w, inp["X"] + 0.02 * rng.standard_normal(inp["X"].shape).astype(np.float32))
    idx_keep = dv.idx.cpu().numpy().copy()
    ref_i = oracle.layer(d, _f64(X1), *Wts, heads=w.heads, Xe=Xe, idx=idx_keep)
    A_keep = tg.host(dv.A)
    Yi, _ = dv.layer(tb.TOMA_REUSE_IDX, X=X1)
    _check_stage("Y reuse idx", Yi, ref_i["Y"], tol)
    assert np.array_equal(dv.idx.cpu().numpy(), idx_keep)
    assert not np.array_equal(tg.host(dv.A), A_keep)          # weights were recomputed
    A1, Z1 = tg.host(dv.A), tg.host(dv.Z)
    X2 = synth.quantize(w, X1 + 0.02 * rng.standard_normal(inp["X"].shape).astype(np.float32))
    ref_a = oracle.layer(d, _f64(X2), *Wts, heads=w.heads, Xe=Xe, idx=idx_keep, AZ=(ref_i["A"], ref_i["Z"]))
    Ya, _ = dv.layer(tb.TOMA_REUSE_A, X=X2)
    _check_stage("Y reuse A", Ya, ref_a["Y"], tol)
    assert np.array_equal(tg.host(dv.A), A1) and np.array_equal(tg.host(dv.Z), Z1)


def test_layer_on_random_shapes(oracle):
    """A seeded sweep of whole layer calls (select, weights, merge, attention, unmerge): grids of one to
    nine regions, tile shapes, widths with heads of 32 or 64, extra tokens, keep ratios, both merge modes
    and both dtypes, against the oracle's layer at the stated tolerances."""
    rng = np.random.default_rng(77)
    done = 0
    while done < 10:
        th, tw = int(rng.choice([2, 4, 6, 8, 16])), int(rng.choice([4, 8, 16, 32]))
        n_loc = th * tw
        if n_loc % 16 or n_loc > 256:
            continue
        gh, gw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        d_loc = int(rng.integers(max(1, n_loc // 8), n_loc // 2 + 1))
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        dh = int(rng.choice([32, 64]))
        heads = int(rng.integers(1, 5))
        T = int(rng.choice([0, 0, 5, 40]))
        w = synth.scaled(W["tiny"], name="randlayer", dtype=dtype, B=2, H=gh * th, W=gw * tw, C=heads * dh, tile_h=th,
                         tile_w=tw, keep=d_loc / n_loc, heads=heads, T_extra=T, index=200 + done)
        if w.d_loc != d_loc:
            continue
        R = w.P if rng.random() < 0.5 else 1
        print(f"[layer random shapes] {dtype} grid {gh}x{gw} tiles of {th}x{tw}, {heads} heads x {dh}, d_loc={d_loc}, "
              f"extra {T}, merge_regions={R}", flush=True)
        inp = synth.make_inputs(w)
        X = _f64(inp["X"])
        Xe = None if inp["X_extra"] is None else _f64(inp["X_extra"])
        Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
        ref = oracle.layer(tg.oracle_desc(oracle, w, R), X, *Wts, heads=w.heads, Xe=Xe)
        dv = tg.Device(w, inp, R)
        Y, Ye = dv.layer(0)
        bad, near, forced = tg.compare_picks(oracle, w, X, dv.idx.cpu().numpy())
        assert not bad
        if np.array_equal(dv.idx.cpu().numpy(), ref["idx"]):   # (a near tie taken the other way changes everything after it)
            _check_stage("Y", Y, ref["Y"], tg.TOL[w.dtype])
            if Ye is not None:
                _check_stage("Y_extra", Ye, ref["Y_extra"], tg.TOL[w.dtype])
        done += 1


@pytest.mark.parametrize("name", ["small_bf16", "tiny"])
def test_greedy_kernel_that_times_its_rounds(cases, name):
    """The profiling variant of the greedy kernel (regions of 256 and of 64 tokens) picks exactly what
    toma_select picks, counts one round per pick in every wave, and its clock sums are plausible (a part
    of a round takes tens to thousands of clocks); other region sizes are refused."""
    w, inp = cases[name]
    print(f"[greedy parts] {name} n_loc={w.n_loc}", flush=True)
    assert w.n_loc in (256, 64)
    dv = tg.Device(w, inp, 1)
    ref = dv.select(gap=False).copy()
    waves = (w.n_loc // 16 + 1) // 2
    parts = torch.full((w.B * w.P, waves, 8), -1, dtype=torch.int64, device="cuda")
    dv.idx.zero_()
    tb.toma_profile_greedy_parts(dv.desc, dv.X, dv.idx, parts, dv.ws)
    torch.cuda.synchronize()
    assert np.array_equal(dv.idx.cpu().numpy(), ref)
    p = parts.cpu().numpy()
    assert np.all(p[:, :, 5] == w.d_loc) and np.all(p[:, :, 7] == 0)
    per_round = p[:, :, :5] / float(w.d_loc)
    assert np.all(per_round > 5) and np.all(per_round < 50000)
    # every column of a region changes at least once (at the first pick), none more often than once per round
    changed = p[:, :, 6].sum(axis=1)
    assert np.all(changed >= w.n_loc) and np.all(changed <= w.n_loc * w.d_loc)
    w2, inp2 = cases["ragged_f32"]
    dv2 = tg.Device(w2, inp2, 1)
    with pytest.raises(tb.TomaError) as e:
        tb.toma_profile_greedy_parts(dv2.desc, dv2.X, dv2.idx, parts, dv2.ws)
    assert e.value.status == 5


@pytest.mark.parametrize("name,tile_local", [("small_bf16", False), ("small_bf16", True), ("ragged_f32", False),
                                             ("extra", False)])
def test_layer_replayed_from_a_graph(cases, name, tile_local):
    """The library only queues kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a layer call can be captured into a graph.  The three kinds of call of the
    reuse schedule (nothing cached, cached idx, cached idx + weights) are captured once each and
    replayed twice along the schedule on drifting tokens, with eager copies and synchronisations
    between the replays; every replay must give the eager call's bits."""
    w, inp = cases[name]
    R = w.P if tile_local else 1
    print(f"[graph] {name} merge_regions={R}", flush=True)
    rng = np.random.default_rng(41)
    Xs = [inp["X"]]
    for _ in range(2):
        Xs.append(synth.quantize(w, Xs[-1] + 0.02 * rng.standard_normal(inp["X"].shape).astype(np.float32)))
    schedule = list(zip((0, tb.TOMA_REUSE_IDX, tb.TOMA_REUSE_A), Xs))
    eager = tg.Device(w, inp, R)
    want = []
    for flags, X in schedule:
        Y, Ye = eager.layer(flags, X=X)
        want.append((Y, Ye, eager.idx.cpu().numpy().copy(), tg.host(eager.Z)))
    dv = tg.Device(w, inp, R)
    side = torch.cuda.Stream()
    graphs = {}
    for flags, _ in schedule:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            tb.toma_layer(dv.desc, dv.attn, flags, dv.X, dv.Xe, dv.idx, dv.A, dv.Z, dv.amap, dv.Wq, dv.Wk, dv.Wv,
                          None, dv.Y, dv.Ye, dv.ws)
        graphs[flags] = g
    for rep in range(2):
        for (flags, X), (Y, Ye, idx, Z) in zip(schedule, want):
            dv.X.copy_(tg.dev(X, w.dtype))
            dv.Y.zero_()
            graphs[flags].replay()
            torch.cuda.synchronize()
            assert np.array_equal(dv.idx.cpu().numpy(), idx), (rep, flags)
            assert np.array_equal(tg.host(dv.Z), Z), (rep, flags)
            assert np.array_equal(tg.host(dv.Y), Y), (rep, flags)
            if Ye is not None:
                assert np.array_equal(tg.host(dv.Ye), Ye), (rep, flags)


@pytest.mark.parametrize("dtype,heads,C,L,T", [("bf16", 2, 256, 200, 0), ("bf16", 1, 32, 77, 5),
                                               ("f32", 2, 128, 130, 0), ("f32", 1, 128, 64, 3),
                                               ("bf16", 10, 640, 256, 1744), ("bf16", 12, 1536, 256, 1244)])
def test_attention_shapes_and_output_projection(oracle, dtype, heads, C, L, T):
    """Head widths 32 / 64 / 128, ragged lengths, extra tokens and the optional W_o.  The two long
    cases (2000 and 1500 tokens over 20 and 24 heads) are sized so that the launch takes workgroups
    of eleven and ten waves, the last one of each head reaching past the end."""
    print(f"[attend] {dtype} heads={heads} C={C} D={L} T={T}", flush=True)
    rng = np.random.default_rng(5)
    # a descriptor whose D equals L: one region of 16 x 16 tokens per 'row', d_loc chosen to fit
    H, Wg, th, tw = 16, 16, 16, 16
    assert L <= 256
    w = synth.scaled(W["tiny"], name="att", dtype=dtype, B=2, H=H, W=Wg, C=C, tile_h=th, tile_w=tw,
                     keep=L / 256, heads=heads, T_extra=T, index=13)
    assert w.D == L
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    Xm = synth.quantize(w, rng.standard_normal((2, L, C)).astype(np.float32))
    Wo = synth.quantize(w, (rng.standard_normal((C, C)) / np.sqrt(C)).astype(np.float32))
    Xe = None if inp["X_extra"] is None else _f64(inp["X_extra"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    O = dv.attend(Xm=Xm)
    _check_stage("O", O, oracle.attend(_f64(Xm), Xe, *Wts, heads=heads), tg.TOL[dtype])
    O2 = dv.attend(Xm=Xm, Wo=tg.dev(Wo, dtype))
    _check_stage("O Wo", O2, oracle.attend(_f64(Xm), Xe, *Wts, heads=heads, Wo=_f64(Wo)), tg.TOL[dtype])


@pytest.mark.parametrize("dtype,head_dim,order", [("bf16", 64, "up"), ("bf16", 64, "down"), ("bf16", 128, "up"),
                                                  ("f32", 64, "up")])
def test_attention_with_drifting_maxima(oracle, dtype, head_dim, order):
    """Scores whose row maxima keep growing along the keys, slowly for some queries and fast for
    others of the same wave (or are largest at the first keys): the streaming softmax has to move
    its reference point per row and rescale what it has accumulated, over 16 key tiles."""
    print(f"[attend drift] {dtype} head_dim={head_dim} {order}", flush=True)
    rng = np.random.default_rng(9)
    C, D, T = head_dim, 256, 768
    w = synth.scaled(W["tiny"], name="drift", dtype=dtype, B=1, H=16, W=16, C=C, tile_h=16, tile_w=16,
                     keep=1.0, heads=1, T_extra=T, index=14)
    assert w.D == D
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    L = D + T
    # token j = a_j e_0 + noise with a_j rising from 1 to about 45: with W_q = W_k = I the score of
    # (i, j) is about a_i a_j, so the maximum of row i grows by about 2.8 a_i per tile of 64 keys
    a = 1.0 + 0.043 * np.arange(L)
    if order == "down":
        a = a[::-1].copy()
    U = 0.05 * rng.standard_normal((1, L, C))
    U[0, :, 0] += a
    U = synth.quantize(w, U.astype(np.float32))
    eye = np.eye(C, dtype=np.float32)
    Wv = synth.quantize(w, (rng.standard_normal((C, C)) / np.sqrt(C)).astype(np.float32))
    dv.Wq.copy_(tg.dev(eye, dtype)); dv.Wk.copy_(tg.dev(eye, dtype)); dv.Wv.copy_(tg.dev(Wv, dtype))
    dv.Xe.copy_(tg.dev(U[:, D:], dtype))
    O = dv.attend(Xm=U[:, :D])
    ref = oracle.attend(_f64(U[:, :D]), _f64(U[:, D:]), _f64(eye), _f64(eye), _f64(Wv), heads=1)
    _check_stage("O", O, ref, tg.TOL[dtype])


@pytest.mark.parametrize("dtype,rows,C,hidden", [("f32", 200, 64, 256), ("bf16", 1000, 128, 512),
                                                  ("bf16", 333, 96, 160), ("bf16", 2 * 2048, 640, 2560)])
def test_mlp_module(oracle, dtype, rows, C, hidden):
    """gelu(X W1) W2 against the oracle: ragged row counts, a width the load-to-LDS GEMM cannot take
    (96 channels in bf16) and the SDXL stage-1 size."""
    rng = np.random.default_rng(5)
    q = lambda a: synth.quantize(synth.scaled(W["tiny"], dtype=dtype), a)
    X = q(rng.standard_normal((rows, C)))
    W1 = q(rng.standard_normal((C, hidden)) / np.sqrt(C))
    W2 = q(rng.standard_normal((hidden, C)) / np.sqrt(hidden))
    print(f"[mlp] {dtype} rows={rows} C={C} hidden={hidden}", flush=True)
    Xd, W1d, W2d = (tg.dev(a, dtype) for a in (X, W1, W2))
    Hb = torch.empty((rows, hidden), dtype=Xd.dtype, device="cuda")
    Out = torch.empty_like(Xd)
    tb.toma_mlp(Xd, W1d, W2d, Hb, Out)
    torch.cuda.synchronize()
    _check_stage("mlp", tg.host(Out), oracle.mlp(_f64(X), _f64(W1), _f64(W2)), tg.TOL[dtype])


def test_block_with_one_merge_and_two_modules(oracle, cases):
    """A block in the ToMA_once style: one merge, attention and the feed-forward module on the merged
    tokens (with the residual paths a transformer block has left out), one unmerge, chained on
    the device and compared with the same chain in the oracle."""
    w, inp = cases["small_bf16"]
    tol = tg.TOL[w.dtype]
    rng = np.random.default_rng(6)
    hidden = 4 * w.C
    W1 = synth.quantize(w, rng.standard_normal((w.C, hidden)) / np.sqrt(w.C))
    W2 = synth.quantize(w, rng.standard_normal((hidden, w.C)) / np.sqrt(hidden))
    X = _f64(inp["X"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, 1)
    idx, _, _ = oracle.select(d, X)
    A, Z, _ = oracle.merge_weights(d, X, idx)
    Xm = oracle.merge(d, X, A, Z)
    O = oracle.attend(Xm, None, *Wts, heads=w.heads)
    F = oracle.mlp(O, _f64(W1), _f64(W2))
    Y_ref = oracle.unmerge(d, A, Z, F)
    dv = tg.Device(w, inp, 1)
    dv.merge(idx=idx)
    dv.attend()
    Hb = torch.empty((w.B * w.D, hidden), dtype=dv.O.dtype, device="cuda")
    F_dev = torch.empty_like(dv.O)
    tb.toma_mlp(dv.O, tg.dev(W1, w.dtype), tg.dev(W2, w.dtype), Hb, F_dev)
    dv.O.copy_(F_dev)
    _check_stage("Y after merge, attention, mlp, unmerge", dv.unmerge(), Y_ref, tol)


@pytest.mark.parametrize("case,t_ctx,c_ctx,use_wo", [("tiny", 9, 32, False), ("small_bf16", 77, 160, True),
                                                      ("small_bf16", 64, 128, False), ("extra", 200, 256, True)])
def test_cross_attention(oracle, cases, case, t_ctx, c_ctx, use_wo):
    """Cross-attention with the [merged ; extra] tokens as queries and a context of another length and
    width (Sec. 5.1, ToMA_once): context widths that take the tiled product and one that does not,
    fewer context tokens than one key tile and more, with and without the output projection."""
    w, inp = cases[case]
    tol = tg.TOL[w.dtype]
    rng = np.random.default_rng(61)
    q = lambda a: synth.quantize(w, np.asarray(a, np.float32))
    L = w.D + w.T_extra
    U = q(rng.standard_normal((w.B, L, w.C)))
    Ctx = q(rng.standard_normal((w.B, t_ctx, c_ctx)))
    Wq = q(rng.standard_normal((w.C, w.C)) / np.sqrt(w.C))
    Wk, Wv = (q(rng.standard_normal((c_ctx, w.C)) / np.sqrt(c_ctx)) for _ in range(2))
    Wo = q(rng.standard_normal((w.C, w.C)) / np.sqrt(w.C)) if use_wo else None
    print(f"[cross] {case}: L={L} C={w.C} heads={w.heads} context {t_ctx} x {c_ctx} Wo={use_wo}", flush=True)
    dv = tg.Device(w, inp, 1)
    dt = w.dtype
    O = torch.empty((w.B, L, w.C), dtype=dv.X.dtype, device="cuda")
    tb.toma_cross_attend(dv.desc, dv.attn, tg.dev(U, dt), tg.dev(Ctx, dt), tg.dev(Wq, dt), tg.dev(Wk, dt), tg.dev(Wv, dt),
                         None if Wo is None else tg.dev(Wo, dt), O, dv.ws)
    torch.cuda.synchronize()
    ref = oracle.cross_attend(_f64(U), _f64(Ctx), _f64(Wq), _f64(Wk), _f64(Wv), w.heads, Wo=None if Wo is None else _f64(Wo))
    _check_stage("O (cross-attention)", tg.host(O), ref, tol)


def test_block_with_one_merge_and_three_modules(oracle, cases):
    """A transformer block in the ToMA_once style (Sec. 5.1): one merge, then self-attention,
    cross-attention to a text-like context and the feed-forward module, all on the merged tokens
    (residual paths left out), one unmerge; chained on the device and in the oracle."""
    w, inp = cases["small_bf16"]
    tol = tg.TOL[w.dtype]
    rng = np.random.default_rng(62)
    q = lambda a: synth.quantize(w, np.asarray(a, np.float32))
    hidden, t_ctx, c_ctx = 4 * w.C, 77, 128
    W1, W2 = q(rng.standard_normal((w.C, hidden)) / np.sqrt(w.C)), q(rng.standard_normal((hidden, w.C)) / np.sqrt(hidden))
    Ctx = q(rng.standard_normal((w.B, t_ctx, c_ctx)))
    Cq = q(rng.standard_normal((w.C, w.C)) / np.sqrt(w.C))
    Ck, Cv = (q(rng.standard_normal((c_ctx, w.C)) / np.sqrt(c_ctx)) for _ in range(2))
    X = _f64(inp["X"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, 1)
    idx, _, _ = oracle.select(d, X)
    A, Z, _ = oracle.merge_weights(d, X, idx)
    Xm = oracle.merge(d, X, A, Z)
    O1 = oracle.attend(Xm, None, *Wts, heads=w.heads)
    O2 = oracle.cross_attend(O1, _f64(Ctx), _f64(Cq), _f64(Ck), _f64(Cv), w.heads)
    F = oracle.mlp(O2, _f64(W1), _f64(W2))
    Y_ref = oracle.unmerge(d, A, Z, F)
    dv = tg.Device(w, inp, 1)
    dt = w.dtype
    dv.merge(idx=idx)
    dv.attend()
    O2d = torch.empty_like(dv.O)
    tb.toma_cross_attend(dv.desc, dv.attn, dv.O, tg.dev(Ctx, dt), tg.dev(Cq, dt), tg.dev(Ck, dt), tg.dev(Cv, dt), None,
                         O2d, dv.ws)
    Hb = torch.empty((w.B * w.D, hidden), dtype=dv.O.dtype, device="cuda")
    tb.toma_mlp(O2d, tg.dev(W1, dt), tg.dev(W2, dt), Hb, dv.O)
    _check_stage("Y after merge, attention, cross-attention, mlp, unmerge", dv.unmerge(), Y_ref, tol)


@pytest.mark.parametrize("tile_local", [False, True])
def test_two_layers_share_one_pattern(oracle, cases, tile_local):
    """Sec. 4.3.2: destinations and merge weights are shared across layers of a block type.  Layer 1
    computes the pattern on its tokens; layer 2 has different tokens and different projections and
    runs on the cached (A, Z, block map) of layer 1; both against the oracle doing the same."""
    w, inp = cases["small_bf16"]
    R = w.P if tile_local else 1
    tol = tg.TOL[w.dtype]
    rng = np.random.default_rng(63)
    q = lambda a: synth.quantize(w, np.asarray(a, np.float32))
    X1 = _f64(inp["X"])
    W1 = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    X2f = q(0.7 * inp["X"] + 0.7 * rng.standard_normal(inp["X"].shape))       # another layer's hidden states
    W2f = [q(rng.standard_normal((w.C, w.C)) / np.sqrt(w.C)) for _ in range(3)]
    d = tg.oracle_desc(oracle, w, R)
    ref1 = oracle.layer(d, X1, *W1, heads=w.heads)
    ref2 = oracle.layer(d, _f64(X2f), *[_f64(a) for a in W2f], heads=w.heads, idx=ref1["idx"], AZ=(ref1["A"], ref1["Z"]))
    dv = tg.Device(w, inp, R)
    Y1, _ = dv.layer(0)
    _check_stage("Y layer 1", Y1, ref1["Y"], tol)
    A1, Z1 = tg.host(dv.A), tg.host(dv.Z)
    dv.Wq, dv.Wk, dv.Wv = (tg.dev(a, w.dtype) for a in W2f)
    Y2, _ = dv.layer(tb.TOMA_REUSE_A, X=X2f)
    _check_stage("Y layer 2 on layer 1's pattern", Y2, ref2["Y"], tol)
    assert np.array_equal(tg.host(dv.A), A1) and np.array_equal(tg.host(dv.Z), Z1)
    # and it differs from what layer 2's own pattern would give (the cache is really what was used)
    own = oracle.layer(d, _f64(X2f), *[_f64(a) for a in W2f], heads=w.heads)
    assert tg.max_rel(own["Y"], ref2["Y"]) > 10 * tol or not np.array_equal(own["idx"], ref1["idx"])


def _clean_rcond(oracle, d, A, Z):
    """A cut-off with no singular value of any region's A~ near it (a value sitting on the cut could
    fall on either side in the two evaluations), and the spectrum's summary."""
    sv, dev = oracle.merge_matrix_spectrum(d, A, Z)
    rel = sv / np.maximum(sv.max(axis=2, keepdims=True), 1e-300)
    for rcond in (1e-2, 3e-3, 3e-2, 1e-3):
        if not np.any((rel > rcond / 6) & (rel < rcond * 6)):
            return rcond, rel, dev
    pytest.skip("no clean gap in the spectrum of the merge matrices")


@pytest.mark.parametrize("case,tile_local", [("tiny", False), ("tiny", True), ("small_bf16", True), ("extra", True),
                                             ("stripe", True)])
def test_pinv_unmerge(oracle, cases, case, tile_local):
    """Moore-Penrose unmerge (Sec. 4.2.2) of the library's own stored (A, Z): against numpy's
    pseudo-inverse of the same matrices in float64, with the cut-off placed in a gap of the spectrum."""
    w, inp = cases[case]
    R = w.P if tile_local else 1
    tol = tg.TOL[w.dtype]
    rng = np.random.default_rng(71)
    d = tg.oracle_desc(oracle, w, R)
    dv = tg.Device(w, inp, R)
    idx, _, _ = oracle.select(d, _f64(inp["X"]))
    A, Z, _ = dv.merge(idx=idx)
    rcond, rel, dev = _clean_rcond(oracle, d, A, np.maximum(Z, 1e-20))
    below = int((rel <= rcond).sum())
    print(f"[pinv] {case} merge_regions={R}: Dr={w.D // R} rcond={rcond:g}; singular values below the cut: {below} of "
          f"{rel.size}; ||A~A~^T - I||_2 max {dev.max():.3f} median {np.median(dev):.3f}", flush=True)
    O = synth.quantize(w, rng.standard_normal((w.B, w.D + w.T_extra, w.C)).astype(np.float32))
    dv.O.copy_(tg.dev(O, w.dtype))
    tb.toma_unmerge_pinv(dv.desc, dv.A, dv.Z, dv.O, rcond, dv.Y, dv.ws)
    torch.cuda.synchronize()
    Y_ref = oracle.unmerge_pinv(d, A, np.maximum(Z, 1e-20), _f64(O), rcond)
    _check_stage("Y (pseudo-inverse unmerge)", tg.host(dv.Y), Y_ref, tol)
    # it is not the transpose unmerge in disguise (the merge matrices here are far from orthonormal)
    assert tg.max_rel(oracle.unmerge(d, A, np.maximum(Z, 1e-20), _f64(O)), Y_ref) > 10 * tol


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_pinv_unmerge_of_rank_deficient_weights(oracle, dtype):
    """Planted merge matrices whose rows are dependent in every way the cut has to handle: a destination
    with no weight (zero row), two destinations with identical rows, and a row that is a combination of
    two others - against numpy's pseudo-inverse (least-squares, minimum-norm answer)."""
    w = synth.scaled(W["tiny"], name="pinv_planted", dtype=dtype, B=2, H=16, W=16, C=64, tile_h=8, tile_w=8, keep=0.5,
                     heads=1, index=27)
    inp = synth.make_inputs(w)
    R, tol = w.P, tg.TOL[dtype]
    rng = np.random.default_rng(72)
    d = tg.oracle_desc(oracle, w, R)
    dv = tg.Device(w, inp, R)
    Dr, Nr = w.d_loc, w.n_loc
    A = (rng.uniform(0.25, 1.0, (w.B, R, Dr, Nr)) * (rng.uniform(size=(w.B, R, Dr, Nr)) < 0.15)).astype(np.float32)
    A[..., np.arange(Dr), np.arange(Dr)] += 0.5              # every destination weighs a source of its own
    A[0, 1, 3] = 0.0                                         # nobody chose destination 3 of region 1
    A[1, 0, 7] = A[1, 0, 2]                                  # identical rows
    A[1, 2, 9] = 0.5 * A[1, 2, 4] + 0.25 * A[1, 2, 5]        # a dependent row (exact in bf16: powers of two)
    A = _f64(synth.quantize(w, A))
    A[1, 2, 9] = 0.5 * A[1, 2, 4] + 0.25 * A[1, 2, 5]
    A = _f64(synth.quantize(w, A.astype(np.float32)))
    Z = A.sum(axis=3).reshape(w.B, w.D)
    dv.plant(A, Z)
    rcond, rel, dev = _clean_rcond(oracle, d, A, np.maximum(Z, 1e-20))
    below = (rel <= rcond).sum(axis=2)
    print(f"[pinv planted] {dtype}: rcond={rcond:g}, singular values below the cut per region: {below.tolist()}", flush=True)
    assert below[0, 1] >= 1 and below[1, 0] >= 1 and below[1, 2] >= 1
    O = synth.quantize(w, rng.standard_normal((w.B, w.D, w.C)).astype(np.float32))
    dv.O.copy_(tg.dev(O, dtype))
    tb.toma_unmerge_pinv(dv.desc, dv.A, dv.Z, dv.O, rcond, dv.Y, dv.ws)
    torch.cuda.synchronize()
    _check_stage("Y (pseudo-inverse unmerge, deficient rank)", tg.host(dv.Y),
                 oracle.unmerge_pinv(d, A, np.maximum(Z, 1e-20), _f64(O), rcond), tol)


@pytest.mark.parametrize("tile_local", [False, True])
@pytest.mark.parametrize("name", list(CASES))
def test_merge_unmerge_with_recomputed_weights(oracle, cases, name, tile_local):
    """Sec. 4.2.1's attention form of the merge: Z, the merged tokens and the unmerged output with
    the weights evaluated on the fly (no A in memory) against the oracle's definitions, and the whole
    layer through the same path (alone and on cached picks)."""
    w, inp = cases[name]
    R = w.P if tile_local else 1
    tol = tg.TOL[w.dtype]
    print(f"[recompute] {name} merge_regions={R}", flush=True)
    X = _f64(inp["X"])
    Xe = None if inp["X_extra"] is None else _f64(inp["X_extra"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, R)
    ref = oracle.layer(d, X, *Wts, heads=w.heads, Xe=Xe)
    dv = tg.Device(w, inp, R)
    Z, Xm = dv.merge_recompute(idx=ref["idx"])
    _check_stage("Z", Z, ref["Z"], tol)
    _check_stage("Xm", Xm, ref["Xm"], tol)
    rng = np.random.default_rng(91)
    O_in = synth.quantize(w, rng.standard_normal((w.B, w.D + w.T_extra, w.C)).astype(np.float32))
    Y = dv.unmerge_recompute(O=O_in)
    _check_stage("Y", Y, oracle.unmerge(d, ref["A"], ref["Z"], _f64(O_in)), tol)
    dv.A.zero_()     # the layer through this path neither reads nor writes A
    Yl, Ye = dv.layer(tb.TOMA_RECOMPUTE_WEIGHTS)
    bad, _, _ = tg.compare_picks(oracle, w, X, dv.idx.cpu().numpy())
    assert not bad
    _check_stage("Y (layer)", Yl, ref["Y"], tol)
    if Ye is not None:
        _check_stage("Y_extra (layer)", Ye, ref["Y_extra"], tol)
    assert not dv.A.any()
    Yi, _ = dv.layer(tb.TOMA_RECOMPUTE_WEIGHTS | tb.TOMA_REUSE_IDX)
    assert np.array_equal(Yi, Yl)
    with pytest.raises(tb.TomaError):
        dv.layer(tb.TOMA_RECOMPUTE_WEIGHTS | tb.TOMA_REUSE_A)


@pytest.mark.parametrize("dtype,tau,C", [("bf16", 0.1, 64), ("bf16", 3.0, 64), ("bf16", 100.0, 64), ("bf16", 0.1, 1024),
                                         ("bf16", 3.0, 1280), ("bf16", 1.0, 3072), ("f32", 0.1, 32), ("f32", 2.0, 320),
                                         ("f32", 8.0, 1024)])
def test_recomputed_weights_skip_only_empty_tiles(oracle, dtype, tau, C):
    """Temperatures from almost one-hot weights (nearly every tile of weights skipped) to almost uniform
    ones (none skipped), and every channel width the kernel is instantiated for: recomputed merge and
    unmerge against the dense definitions."""
    big = C > 640
    w = synth.scaled(W["tiny"], name="rc", dtype=dtype, B=2 if not big else 1, H=32 if big else 64, W=32 if big else 64,
                     C=C, tile_h=16, tile_w=16, keep=0.5, heads=max(1, C // 64), tau=tau, index=29)
    print(f"[recompute tiles] {dtype} tau={tau} C={C} N={w.N} D={w.D}", flush=True)
    inp = synth.make_inputs(w)
    tol = tg.TOL[dtype]
    X = _f64(inp["X"])
    d = tg.oracle_desc(oracle, w, 1)
    idx, _, _ = oracle.select(d, X)
    A_ref, Z_ref, _ = oracle.merge_weights(d, X, idx)
    dv = tg.Device(w, inp, 1)
    Z, Xm = dv.merge_recompute(idx=idx)
    _check_stage("Z", Z, Z_ref, tol)
    _check_stage("Xm", Xm, oracle.merge(d, X, A_ref, Z_ref), tol)
    rng = np.random.default_rng(92)
    O_in = synth.quantize(w, rng.standard_normal((w.B, w.D, w.C)).astype(np.float32))
    _check_stage("Y", dv.unmerge_recompute(O=O_in), oracle.unmerge(d, A_ref, Z_ref, _f64(O_in)), tol)


def test_binding_reports_errors_on_device():
    w, = (W["tiny"],)
    inp = synth.make_inputs(w)
    dv = tg.Device(w, inp, 1)
    with pytest.raises(tb.TomaError) as e:
        tb.toma_select(dv.desc, dv.X, dv.idx, None, None, dv.ws[:256])
    assert e.value.status == 4
    with pytest.raises(tb.TomaError) as e:
        tb.toma_unmerge(dv.desc, dv.A, dv.Z, dv.amap, dv.O[:, :10].contiguous(), dv.Y, dv.ws)
    assert e.value.status == 2
