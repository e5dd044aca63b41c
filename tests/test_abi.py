"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and turns bad arguments into status codes before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2509_10918_amd import binding as tb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "toma.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(toma_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = _declared()
    assert sorted(names) == sorted(tb.EXPORTS)
    L = tb.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert tb.status_string(0) == "ok"
    assert len({tb.status_string(i) for i in range(7)}) == 7


def _d(**kw):
    base = dict(B=2, H=64, W=64, C=640, tile_h=16, tile_w=16, d_loc=128, merge_regions=1, tau=0.1, dtype="bf16")
    base.update(kw)
    return tb.make_desc(**base)


def test_workspace_bytes_and_shape_errors():
    a = tb.toma_attn_desc(10, 64, 0)
    n = tb.toma_workspace_bytes(_d(), a)
    assert n > 0 and n % 256 == 0
    assert tb.toma_workspace_bytes(_d(), None) > 0
    assert tb.toma_workspace_bytes(_d(tile_h=15), a) == 0          # does not divide the grid
    assert tb.toma_workspace_bytes(_d(d_loc=257), a) == 0           # more destinations than tokens
    assert tb.toma_workspace_bytes(_d(merge_regions=4), a) == 0     # neither 1 nor P
    assert tb.toma_workspace_bytes(_d(C=650), a) == 0               # width not a multiple of 32
    assert tb.toma_workspace_bytes(_d(tile_h=32, tile_w=32), a) > 0   # regions of 1024 tokens: the large-region selection
    assert tb.toma_workspace_bytes(_d(tile_h=64, tile_w=64), a) == 0  # region larger than 2048 tokens
    assert tb.toma_workspace_bytes(_d(tau=0.0), a) == 0
    assert tb.toma_workspace_bytes(_d(), tb.toma_attn_desc(10, 32, 0)) == 0   # heads * head_dim != C
    assert tb.toma_workspace_bytes(None, None) == 0


def test_argument_errors_are_reported_before_any_launch():
    L = tb.lib()
    d = _d()
    a = tb.toma_attn_desc(10, 64, 0)
    dp, ap = ctypes.addressof(d), ctypes.addressof(a)
    need = tb.toma_workspace_bytes(d, a)
    ws = 256 * 1024          # fake but aligned addresses: nothing is dereferenced on these paths
    x = 1 << 20
    assert L.toma_select(None, x, x, None, None, ws, need, None) == 1
    assert L.toma_select(dp, None, x, None, None, ws, need, None) == 1
    assert L.toma_select(dp, x, x, None, None, None, need, None) == 1
    assert L.toma_select(dp, x, x, None, None, ws + 16, need, None) == 3
    assert L.toma_select(dp, x + 8, x, None, None, ws, need, None) == 3
    assert L.toma_select(dp, x, x, x, x + 2, ws, need, None) == 3                # misaligned gap output
    assert L.toma_select(dp, x, x, None, None, ws, tb.toma_workspace_bytes(d, None) - 1, None) == 4
    assert L.toma_layer(dp, ap, 0, x, None, x, x, x, x, x, x, x, None, x, None, ws, need - 1, None) == 4
    bad = _d(tile_w=48)
    assert L.toma_select(ctypes.addressof(bad), x, x, None, None, ws, need, None) == 2
    big = _d(tile_h=64, tile_w=64, d_loc=2048)   # a region of 4096 tokens: beyond the selection kernels
    assert L.toma_select(ctypes.addressof(big), x, x, None, None, ws, need, None) == 5
    assert L.toma_merge(dp, x, x, None, x, x, x, ws, need, None) == 1
    assert L.toma_merge_cached(dp, x, x, x, x, None, ws, need, None) == 1
    # the block map travels with (A, Z): required exactly when the shape uses one (stale-cache misuse
    # that the host can see: a missing or misaligned map)
    assert tb.toma_map_bytes(d) > 0 and tb.toma_map_bytes(d) % 256 == 0
    assert L.toma_merge(dp, x, x, x, x, None, x, ws, need, None) == 1
    assert L.toma_merge_cached(dp, x, x, x, None, x, ws, need, None) == 1
    assert L.toma_merge_cached(dp, x, x, x, x + 4, x, ws, need, None) == 3
    assert L.toma_unmerge(dp, x, x, None, x, 2048, x, ws, need, None) == 1
    assert L.toma_layer(dp, ap, 2, x, None, x, x, x, None, x, x, x, None, x, None, ws, need, None) == 1
    assert L.toma_map_build(dp, x, None, None) == 1
    assert L.toma_map_build(dp, None, x, None) == 1
    small = _d(H=16, W=16, tile_h=8, tile_w=8, d_loc=32)     # short products: no map, NULL is fine
    assert tb.toma_map_bytes(small) == 0
    assert L.toma_merge_cached(ctypes.addressof(small), x, x, x, None, None, ws, need, None) == 1   # (Xm missing)
    assert tb.toma_map_bytes(None) == 0
    assert L.toma_attend(dp, None, x, None, x, x, x, None, x, ws, need, None) == 1
    assert L.toma_attend(dp, ap, x, x, x, x, x, None, x, ws, need, None) == 1   # extra tokens given, t_extra == 0
    assert L.toma_unmerge(dp, x, x, x, x, 100, x, ws, need, None) == 2          # fewer rows than D
    assert L.toma_layer(dp, ap, 16, x, None, x, x, x, x, x, x, x, None, x, None, ws, need, None) == 5
    assert L.toma_layer(dp, ap, 0, x, None, None, x, x, x, x, x, x, None, x, None, ws, need, None) == 1
    # cross-attention: context shape and size limits, null checks
    assert L.toma_cross_attend(dp, ap, x, x, 77, 2048, x, x, x, None, None, ws, need, None) == 1
    assert L.toma_cross_attend(dp, ap, x, x, 0, 2048, x, x, x, None, x, ws, need, None) == 2
    assert L.toma_cross_attend(dp, ap, x, x, 77, 2050, x, x, x, None, x, ws, need, None) == 5
    assert L.toma_cross_attend(dp, ap, x, x, 5000, 2048, x, x, x, None, x, ws, need, None) == 5   # more context than queries
    assert L.toma_cross_attend(dp, None, x, x, 77, 2048, x, x, x, None, x, ws, need, None) == 1
    # Moore-Penrose unmerge: cut-off range, region size limit
    assert L.toma_unmerge_pinv(dp, x, x, x, 2048, ctypes.c_float(1e-2), x, ws, need, None) == 5   # 2048 destinations in one region
    tl = _d(merge_regions=16)
    tlp, need_tl = ctypes.addressof(tl), tb.toma_workspace_bytes(tl, a)
    assert L.toma_unmerge_pinv(tlp, x, x, x, 2048, ctypes.c_float(1.5), x, ws, need_tl, None) == 2
    assert L.toma_unmerge_pinv(tlp, x, x, x, 100, ctypes.c_float(1e-2), x, ws, need_tl, None) == 2
    assert L.toma_unmerge_pinv(tlp, x, None, x, 2048, ctypes.c_float(1e-2), x, ws, need_tl, None) == 1
    assert L.toma_unmerge_pinv(tlp, x, x, x, 2048, ctypes.c_float(1e-2), x, ws, tb.toma_workspace_bytes(tl, None) - 1, None) == 4
    # recomputed weights: cache size, null and alignment checks, flag combinations of the layer
    assert tb.toma_recompute_cache_bytes(d) > 2 * 4096 * 4 and tb.toma_recompute_cache_bytes(None) == 0
    assert L.toma_merge_recompute(dp, x, x, x, None, x, ws, need, None) == 1
    assert L.toma_merge_recompute(dp, x, x, x, x + 16, x, ws, need, None) == 3
    assert L.toma_unmerge_recompute(dp, x, x, x, x, x, 100, x, ws, need, None) == 2
    assert L.toma_unmerge_recompute(dp, x, x, None, x, x, 2048, x, ws, need, None) == 1
    assert L.toma_layer(dp, ap, 4 | 2, x, None, x, x, x, x, x, x, x, None, x, None, ws, need, None) == 5
    assert L.toma_layer(dp, ap, 8, x, None, x, x, x, x, x, x, x, None, x, None, ws, need, None) == 5
    # feed-forward module: dtype, shape, divisibility, null and alignment checks
    assert L.toma_mlp(1, 4096, 640, 2560, x, x, x, x, None, None) == 1
    assert L.toma_mlp(1, 0, 640, 2560, x, x, x, x, x, None) == 2
    assert L.toma_mlp(1, 4096, 640, 2500, x, x, x, x, x, None) == 5
    assert L.toma_mlp(7, 4096, 640, 2560, x, x, x, x, x, None) == 5
    assert L.toma_mlp(0, 4096, 640, 2560, x, x + 4, x, x, x, None) == 3
    # the timing variant of the selection: same checks as toma_select, plus the region sizes it exists for
    need_s = tb.toma_workspace_bytes(d, None)
    assert L.toma_profile_greedy_parts(dp, x, x, None, ws, need_s, None) == 1
    assert L.toma_profile_greedy_parts(dp, None, x, x, ws, need_s, None) == 1
    assert L.toma_profile_greedy_parts(dp, x, x, x + 4, ws, need_s, None) == 3
    assert L.toma_profile_greedy_parts(dp, x, x, x, ws, need_s - 1, None) == 4
    other = _d(tile_h=8, tile_w=16, d_loc=64)   # regions of 128 tokens
    assert L.toma_profile_greedy_parts(ctypes.addressof(other), x, x, x, ws, need_s, None) == 5


def test_binding_raises_with_status():
    with pytest.raises(tb.TomaError) as e:
        tb._check(4, "toma_select")
    assert e.value.status == 4 and "workspace" in str(e.value)


@pytest.mark.parametrize("H,W,th,tw,R", [(8, 12, 4, 4, 1), (8, 12, 4, 4, 6), (6, 8, 3, 8, 1), (16, 16, 16, 16, 1)])
def test_column_order_helper_of_the_gpu_tests(H, W, th, tw, R):
    """The GPU tests compare the stored A with the oracle's through toma_gpu.source_tokens, which restates
    the documented column order (toma_merge in toma.h): with one merge region, column s is token
    s % N_loc of selection region s / N_loc; with one merge region per selection region, token s of
    that region (Sec. 4.3.1's region / local index).  Checked here against the definition written out."""
    import toma_gpu as tg
    d = tb.make_desc(1, H, W, 32, th, tw, 1, R, 0.1, "f32")
    got = tg.source_tokens(d)
    pw, n_loc = W // tw, th * tw
    P = (H // th) * pw
    want = []
    for p in range(P):
        for l in range(n_loc):
            r, c = (p // pw) * th + l // tw, (p % pw) * tw + l % tw
            want.append(r * W + c)
    assert got.shape == (R, H * W // R)
    assert got.reshape(-1).tolist() == want
    assert sorted(want) == list(range(H * W))        # every token exactly once


def test_profile_map_product_is_host_arithmetic():
    """The tile a product will run with comes from the descriptor alone (no GPU): merge and unmerge of
    the SDXL stage-1 workload take the tiled path; its weights are made in one pass, so there is no
    write-pass tile to report, while the Flux block's weights take two passes and have one."""
    from paper_2509_10918_amd import synth
    w = synth.WORKLOADS["sdxl1"]
    d = tb.make_desc(w.B, w.H, w.W, w.C, w.tile_h, w.tile_w, w.d_loc, 1, w.tau, w.dtype)
    for which in (0, 1):
        bm, bn, split = tb.toma_profile_map_product(d, which)
        assert bm in (64, 128, 256) and bn in (64, 128, 256) and split >= 1
    assert tb.toma_profile_map_product(d, 2) is None
    assert tb.toma_profile_map_product(d, 3) is None
    f = synth.WORKLOADS["flux"]
    df = tb.make_desc(f.B, f.H, f.W, f.C, f.tile_h, f.tile_w, f.d_loc, 1, f.tau, f.dtype)
    bm, bn, split = tb.toma_profile_map_product(df, 2)
    assert bm in (64, 128, 256) and bn in (64, 128, 256) and split == 1
