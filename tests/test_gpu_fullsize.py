"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration bench.py
times (toma_layer through the C ABI).  SDXL stage 1 / stage 2 and the Flux-shaped block are checked
against the complete fp64 oracle; the 128 x 128 high-resolution sequence is checked completely at step
0 (global merge) and on sampled regions along its reuse schedule (global and region-local merge)."""
import numpy as np
import pytest
import torch

from paper_2509_10918_amd import binding as tb
from paper_2509_10918_amd import synth

import toma_gpu as tg

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def _report(name, got, ref, tol):
    err = tg.max_rel(got, ref)
    ex = tg.elem_excess(got, ref, tol)
    print(f"  {name}: max|err|/max|ref| = {err:.3e} (tol {tol:g}); element-wise excess {ex:.3f}", flush=True)
    assert np.all(np.isfinite(got)) and err <= tol, name
    assert ex <= tg.MAX_ELEM_EXCESS, name


@pytest.mark.timeout(900)
@pytest.mark.parametrize("tile_local", [False, True])
@pytest.mark.parametrize("name", ["sdxl1", "sdxl2", "flux", "sdxl1_stripe", "sdxl1_4regions"])
def test_full_workload_layer(oracle, name, tile_local):
    w = W[name]
    R = w.P if tile_local else 1
    tol = tg.TOL[w.dtype]
    print(f"[full] {name} merge_regions={R}: B={w.B} N={w.N} C={w.C} D={w.D} heads={w.heads} T={w.T_extra}",
          flush=True)
    inp = synth.make_inputs(w)
    X, Xe = _f64(inp["X"]), _f64(inp["X_extra"])
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, R)
    ref = oracle.layer(d, X, *Wts, heads=w.heads, Xe=Xe)
    print(f"  oracle done; destinations with Z < 1e-20: {ref['clamps']}", flush=True)
    dv = tg.Device(w, inp, R)
    Y, Ye = dv.layer(0)
    bad, near, forced = tg.compare_picks(oracle, w, X, dv.idx.cpu().numpy())
    print(f"  near-tie steps {near}, regions verified teacher-forced {forced}, mismatching {bad}", flush=True)
    assert not bad
    _report("Z", tg.host(dv.Z), ref["Z"], tol)
    _report("Y", Y, ref["Y"], tol)
    if Ye is not None:
        _report("Y_extra", Ye, ref["Y_extra"], tol)
    # stage-isolated merge at full size (fed the oracle's picks)
    _, Z, Xm = dv.merge(idx=ref["idx"])
    _report("Xm", Xm, ref["Xm"], tol)
    # cached variants reproduce the full call bit for bit on unchanged tokens
    Yi, _ = dv.layer(tb.TOMA_REUSE_IDX)
    Ya, _ = dv.layer(tb.TOMA_REUSE_A)
    assert np.array_equal(Yi, Y) and np.array_equal(Ya, Y)
    # the same layer with the weights recomputed inside merge and unmerge instead of stored (Sec. 4.2.1)
    Yr, Yre = dv.layer(tb.TOMA_RECOMPUTE_WEIGHTS | tb.TOMA_REUSE_IDX)
    _report("Z (recomputed weights)", tg.host(dv.Z), ref["Z"], tol)
    _report("Y (recomputed weights)", Yr, ref["Y"], tol)
    if Yre is not None:
        _report("Y_extra (recomputed weights)", Yre, ref["Y_extra"], tol)


@pytest.mark.timeout(1500)
def test_hires_reuse_sequence_global(oracle):
    """The 128 x 128 grid with ONE merge region per sample (A is 537 MB: two-pass weights with the
    empty tiles skipped, the block map of a cached A) along its reuse schedule (Sec. 4.3.2): step 0 is
    checked completely against the oracle's layer; steps 1 (everything cached), 2 (cached picks, new
    weights) and 5 (new picks) are checked for exact picks, Z, and Y on the tokens of four sampled
    regions per sample.  For those the oracle evaluates the attention only on the destinations that
    weigh on a sampled token at all (weight above 1e-30; the rest contribute less than 1e-26 of a
    value) and sums the unmerge for the sampled tokens directly from its definition."""
    w = W["hires"]
    tol = tg.TOL[w.dtype]
    print(f"[full] hires, global merge: N={w.N} D={w.D} (A is {w.B * w.D * w.N * 2 / 1e6:.0f} MB)", flush=True)
    inp = synth.make_inputs(w)
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, 1)
    dv = tg.Device(w, inp, 1)
    _, _, token_of = oracle.region_map(w.H, w.W, w.tile_h, w.tile_w)
    rng = np.random.default_rng(14)
    regions = [sorted(rng.choice(w.P, 4, replace=False).tolist()) for _ in range(w.B)]
    idx = A = Z = None
    for t, (sel, rew) in enumerate(synth.reuse_schedule(w)):
        if t > 5:
            break
        flags = 0 if sel else (tb.TOMA_REUSE_IDX if rew else tb.TOMA_REUSE_A)
        Xt = inp["X_steps"][t]
        Y, _ = dv.layer(flags, X=Xt)
        print(f"[hires global] step {t}: reselect={sel} reweight={rew}", flush=True)
        if t not in (0, 1, 2, 5):
            continue
        X = _f64(Xt)
        if t == 0:
            ref = oracle.layer(d, X, *Wts, heads=w.heads)
            print(f"  oracle done; destinations with Z < 1e-20: {ref['clamps']}", flush=True)
            idx, A, Z = ref["idx"], ref["A"], ref["Z"]
            assert np.array_equal(dv.idx.cpu().numpy(), idx)
            _report("Z step 0", tg.host(dv.Z), Z, tol)
            _report("Y step 0", Y, ref["Y"], tol)
            # the same step with the weights recomputed instead of stored (no half-gigabyte A)
            A_keep = dv.A.clone()
            Yr, _ = dv.layer(tb.TOMA_RECOMPUTE_WEIGHTS | tb.TOMA_REUSE_IDX, X=Xt)
            _report("Y step 0 (recomputed weights)", Yr, ref["Y"], tol)
            assert torch.equal(dv.A, A_keep)
            del ref, A_keep
            continue
        if sel:
            idx, _, _ = oracle.select(d, X)
            assert np.array_equal(dv.idx.cpu().numpy(), idx)
        if rew:
            A, Z, _ = oracle.merge_weights(d, X, idx)
            _report(f"Z step {t}", tg.host(dv.Z), Z, tol)
        Xm = oracle.merge(d, X, A, Z)
        print(f"  oracle weights / merge done", flush=True)
        Zc = np.maximum(Z, 1e-20)
        for b in range(w.B):
            toks = np.concatenate([token_of[p] for p in regions[b]])
            Ab = A[b, 0][:, toks]                                   # [D, sampled tokens]
            dests = np.nonzero(Ab.max(axis=1) > 1e-30)[0]
            rows = (b * w.D + dests).astype(np.int32)
            O_rows = oracle.attend_rows(Xm, None, *Wts, heads=w.heads, rows=rows)
            Y_ref = (Ab[dests] / Zc[b, dests, None]).T @ O_rows      # Sec. 4.2.2 on the sampled tokens
            print(f"  sample {b}: {len(dests)} destinations weigh on the {len(toks)} sampled tokens", flush=True)
            _report(f"Y step {t} sample {b}", Y[b, toks], Y_ref, tol)


@pytest.mark.timeout(1200)
def test_hires_reuse_sequence_tile(oracle):
    """Ten drifting steps, destinations re-selected every 5 steps, weights recomputed every 2
    (Sec. 4.3.2); region-local merge.  The oracle follows the same schedule; attention and unmerge
    are checked on the destinations / tokens of four sampled regions per sample."""
    w = W["hires"]
    R, tol = w.P, tg.TOL[w.dtype]
    inp = synth.make_inputs(w)
    Wts = [_f64(inp[k]) for k in ("Wq", "Wk", "Wv")]
    d = tg.oracle_desc(oracle, w, R)
    dv = tg.Device(w, inp, R)
    _, _, token_of = oracle.region_map(w.H, w.W, w.tile_h, w.tile_w)
    rng = np.random.default_rng(4)
    regions = [sorted(rng.choice(w.P, 4, replace=False).tolist()) for _ in range(w.B)]
    rows = np.array([b * w.D + p * w.d_loc + k for b in range(w.B) for p in regions[b] for k in range(w.d_loc)],
                    np.int32)
    idx = A = Z = None
    check_at = {0, 1, 2, 5, 6, 9}
    for t, (sel, rew) in enumerate(synth.reuse_schedule(w)):
        flags = 0 if sel else (tb.TOMA_REUSE_IDX if rew else tb.TOMA_REUSE_A)
        Xt = inp["X_steps"][t]
        Y, _ = dv.layer(flags, X=Xt)
        print(f"[hires] step {t}: reselect={sel} reweight={rew}", flush=True)
        X = _f64(Xt)
        if sel:
            idx, _, _ = oracle.select(d, X)
            assert np.array_equal(dv.idx.cpu().numpy(), idx)
        if rew:
            A, Z, _ = oracle.merge_weights(d, X, idx)
        if t not in check_at:
            continue
        Xm = oracle.merge(d, X, A, Z)
        O_rows = oracle.attend_rows(Xm, None, *Wts, heads=w.heads, rows=rows)
        O = np.zeros((w.B, w.D, w.C))
        O.reshape(-1, w.C)[rows] = O_rows
        Y_ref = oracle.unmerge(d, A, Z, O)
        for b in range(w.B):
            toks = np.concatenate([token_of[p] for p in regions[b]])
            _report(f"Y step {t} sample {b}", Y[b, toks], Y_ref[b, toks], tol)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["sdxl1", "flux"])
def test_pinv_unmerge_full_size(oracle, name):
    """Moore-Penrose unmerge at the benchmark sizes with region-local merge (128 / 64 destinations per
    region): the library's stored (A, Z) against numpy's pseudo-inverse, and the spectrum that
    Sec. 4.2.2's orthonormality argument is about, as found on these inputs."""
    w = W[name]
    R, tol = w.P, tg.TOL[w.dtype]
    inp = synth.make_inputs(w)
    d = tg.oracle_desc(oracle, w, R)
    dv = tg.Device(w, inp, R)
    idx = dv.select()
    A, Z, _ = dv.merge()
    sv, dev = oracle.merge_matrix_spectrum(d, A, np.maximum(Z, 1e-20))
    rel = sv / sv.max(axis=2, keepdims=True)
    rcond = 1e-2
    assert not np.any((rel > rcond / 6) & (rel < rcond * 6)), "a singular value sits near the cut"
    print(f"[pinv full] {name}: {int((rel <= rcond).sum())} of {rel.size} singular values below {rcond:g} "
          f"({int((Z < 1e-20).sum())} destinations without weight); ||A~A~^T - I||_2 max {dev.max():.3f} "
          f"median {np.median(dev):.3f} min {dev.min():.3f}", flush=True)
    rng = np.random.default_rng(81)
    O = synth.quantize(w, rng.standard_normal((w.B, w.D + w.T_extra, w.C)).astype(np.float32))
    dv.O.copy_(tg.dev(O, w.dtype))
    tb.toma_unmerge_pinv(dv.desc, dv.A, dv.Z, dv.O, rcond, dv.Y, dv.ws)
    torch.cuda.synchronize()
    _report("Y (pseudo-inverse unmerge)", tg.host(dv.Y), oracle.unmerge_pinv(d, A, np.maximum(Z, 1e-20), _f64(O), rcond), tol)
