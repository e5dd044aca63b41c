"""ctypes front end of the fp64 CPU oracle (toma_oracle.c).  Test infrastructure.

All arrays are numpy float64 / int32, dense and row-major.  Each wrapper only marshals arguments;
what is computed, and which passage of the paper it follows, is stated in the C source.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)


class OracleDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("C", ctypes.c_int32), ("tile_h", ctypes.c_int32), ("tile_w", ctypes.c_int32),
                ("d_loc", ctypes.c_int32), ("merge_regions", ctypes.c_int32),
                ("scale", ctypes.c_double), ("sim_bits", ctypes.c_int32)]


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        _lib.toma_oracle_fl_value.restype = ctypes.c_double
        _lib.toma_oracle_check_picks.restype = ctypes.c_int
    return _lib


def _d(a):
    return a.ctypes.data_as(_dp)


def _i(a):
    return a.ctypes.data_as(_ip)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


SIM_BITS = 30  # similarities are decided on a 2^-30 grid (see toma_oracle.c)


def make_desc(B, H, W, C, tile_h, tile_w, d_loc, merge_regions, tau, sim_bits=SIM_BITS, scale=None):
    if H % tile_h or W % tile_w:
        raise ValueError("tiles must divide the grid")
    P = (H // tile_h) * (W // tile_w)
    if merge_regions not in (1, P):
        raise ValueError("merge_regions must be 1 or P")
    if not 1 <= d_loc <= tile_h * tile_w:
        raise ValueError("d_loc out of range")
    return OracleDesc(B, H, W, C, tile_h, tile_w, d_loc, merge_regions,
                      float(scale if scale is not None else 1.0 / tau), int(sim_bits))


def n_regions(d):
    return (d.H // d.tile_h) * (d.W // d.tile_w)


def region_map(H, W, tile_h, tile_w):
    N = H * W
    region = np.empty(N, np.int32)
    local = np.empty(N, np.int32)
    token_of = np.empty(N, np.int32)
    lib().toma_oracle_region_map(H, W, tile_h, tile_w, _i(region), _i(local), _i(token_of))
    P = (H // tile_h) * (W // tile_w)
    return region, local, token_of.reshape(P, tile_h * tile_w)


def cosine(X, round_bits=0):
    X = _f64(X)
    n, C = X.shape
    rows = np.arange(n, dtype=np.int32)
    S = np.empty((n, n), np.float64)
    lib().toma_oracle_cosine(_d(X), _i(rows), n, C, int(round_bits), _d(S))
    return S


def fl_value(S, subset):
    S = _f64(S)
    subset = _i32(subset)
    return lib().toma_oracle_fl_value(_d(S), S.shape[0], _i(subset), len(subset))


def greedy_fl(S, k):
    S = _f64(S)
    picks = np.empty(k, np.int32)
    gains = np.empty(k, np.float64)
    gaps = np.empty(k, np.float64)
    lib().toma_oracle_greedy_fl(_d(S), S.shape[0], k, _i(picks), _d(gains), _d(gaps))
    return picks, gains, gaps


def greedy_direct(S, k):
    S = _f64(S)
    picks = np.empty(k, np.int32)
    gains = np.empty(k, np.float64)
    lib().toma_oracle_greedy_direct(_d(S), S.shape[0], k, _i(picks), _d(gains))
    return picks, gains


def check_picks(S, picks):
    S = _f64(S)
    picks = _i32(picks)
    k = len(picks)
    deficit = np.zeros(k, np.float64)
    is_first = np.zeros(k, np.int32)
    bad = lib().toma_oracle_check_picks(_d(S), S.shape[0], k, _i(picks), _d(deficit), _i(is_first))
    return bad, deficit, is_first


def select(d, X):
    X = _f64(X)
    P = n_regions(d)
    assert X.shape == (d.B, d.H * d.W, d.C)
    idx = np.empty((d.B, P, d.d_loc), np.int32)
    gain = np.empty((d.B, P, d.d_loc), np.float64)
    gap = np.empty((d.B, P, d.d_loc), np.float64)
    lib().toma_oracle_select(ctypes.byref(d), _d(X), _i(idx), _d(gain), _d(gap))
    return idx, gain, gap


def merge_weights(d, X, idx):
    X = _f64(X)
    idx = _i32(idx)
    P = n_regions(d)
    N, D, R = d.H * d.W, P * d.d_loc, d.merge_regions
    A = np.empty((d.B, R, D // R, N // R), np.float64)
    Z = np.empty((d.B, D), np.float64)
    clamps = ctypes.c_int64(0)
    lib().toma_oracle_merge_weights(ctypes.byref(d), _d(X), _i(idx), _d(A), _d(Z), ctypes.byref(clamps))
    return A, Z, clamps.value


def merge(d, X, A, Z):
    X, A, Z = _f64(X), _f64(A), _f64(Z)
    D = n_regions(d) * d.d_loc
    Xm = np.empty((d.B, D, d.C), np.float64)
    lib().toma_oracle_merge(ctypes.byref(d), _d(X), _d(A), _d(Z), _d(Xm))
    return Xm


def attend(Xm, Xe, Wq, Wk, Wv, heads, Wo=None):
    Xm = _f64(Xm)
    B, D, C = Xm.shape
    T = 0 if Xe is None else Xe.shape[1]
    Xe_p = None if Xe is None else _f64(Xe)
    Wq, Wk, Wv = _f64(Wq), _f64(Wk), _f64(Wv)
    Wo_p = None if Wo is None else _f64(Wo)
    O = np.empty((B, D + T, C), np.float64)
    lib().toma_oracle_attend(B, D, T, C, heads, _d(Xm), None if Xe_p is None else _d(Xe_p),
                             _d(Wq), _d(Wk), _d(Wv), None if Wo_p is None else _d(Wo_p), _d(O))
    return O


def attend_rows(Xm, Xe, Wq, Wk, Wv, heads, rows):
    """Attention output for the listed rows only (rows index the B*(D+T) token rows)."""
    Xm = _f64(Xm)
    B, D, C = Xm.shape
    T = 0 if Xe is None else Xe.shape[1]
    Xe_p = None if Xe is None else _f64(Xe)
    Wq, Wk, Wv = _f64(Wq), _f64(Wk), _f64(Wv)
    rows = _i32(rows)
    out = np.empty((len(rows), C), np.float64)
    lib().toma_oracle_attend_rows(B, D, T, C, heads, _d(Xm), None if Xe_p is None else _d(Xe_p),
                                  _d(Wq), _d(Wk), _d(Wv), _i(rows), len(rows), _d(out))
    return out


def cross_attend(U, Ctx, Wq, Wk, Wv, heads, Wo=None):
    """Cross-attention: queries from U [B, Lq, C], keys and values from Ctx [B, Tc, Cc]."""
    U, Ctx = _f64(U), _f64(Ctx)
    B, Lq, C = U.shape
    _, Tc, Cc = Ctx.shape
    Wq, Wk, Wv = _f64(Wq), _f64(Wk), _f64(Wv)
    assert Wq.shape == (C, C) and Wk.shape == (Cc, C) and Wv.shape == (Cc, C)
    Wo_p = None if Wo is None else _f64(Wo)
    O = np.empty((B, Lq, C), np.float64)
    lib().toma_oracle_cross_attend(B, Lq, Tc, C, Cc, heads, _d(U), _d(Ctx), _d(Wq), _d(Wk), _d(Wv),
                                   None if Wo_p is None else _d(Wo_p), _d(O))
    return O


def mlp(X, W1, W2):
    """gelu(X W1) W2 on the rows of X (any leading shape)."""
    X, W1, W2 = _f64(X), _f64(W1), _f64(W2)
    C, hidden = W1.shape
    rows = X.size // C
    out = np.empty_like(X)
    lib().toma_oracle_mlp(rows, C, hidden, _d(X), _d(W1), _d(W2), _d(out))
    return out


def unmerge(d, A, Z, O):
    A, Z, O = _f64(A), _f64(Z), _f64(O)
    N = d.H * d.W
    Y = np.empty((d.B, N, d.C), np.float64)
    lib().toma_oracle_unmerge(ctypes.byref(d), _d(A), _d(Z), _d(O), O.shape[1], _d(Y))
    return Y


def _merge_region_tokens(d):
    """[R, Nr] grid index of source s of merge region rho, in the order the oracle's A has its columns."""
    N, R = d.H * d.W, d.merge_regions
    if R == 1:
        return np.arange(N, dtype=np.int64).reshape(1, N)
    _, _, token_of = region_map(d.H, d.W, d.tile_h, d.tile_w)
    return token_of.astype(np.int64)


def unmerge_pinv(d, A, Z, O, rcond):
    """Sec. 4.2.2, first display: X'_unmerged = A~^+ X' with A~^+ the Moore-Penrose pseudo-inverse of the
    row-normalised merge matrix A~ = A / Z of each merge region (for rows of full rank this is
    A~^T (A~ A~^T)^-1, the closed form the paper prints).  The pseudo-inverse is numpy's
    (SVD; singular values <= rcond * largest are treated as zero - the paper does not name a cut-off,
    so it is an argument).  O is [B, o_rows, C], rows [0, D) are used; Y is [B, N, C] in grid order."""
    A, Z, O = _f64(A), _f64(Z), _f64(O)
    R = d.merge_regions
    D, Dr = A.shape[1] * A.shape[2], A.shape[2]
    tok = _merge_region_tokens(d)
    Y = np.zeros((d.B, d.H * d.W, O.shape[2]), np.float64)
    for b in range(d.B):
        for rho in range(R):
            z = np.maximum(Z[b, rho * Dr:(rho + 1) * Dr], 1e-20)
            At = A[b, rho] / z[:, None]
            Y[b, tok[rho]] = np.linalg.pinv(At, rcond=rcond) @ O[b, rho * Dr:(rho + 1) * Dr]
    return Y


def merge_matrix_spectrum(d, A, Z):
    """Per (sample, merge region): singular values of A~ = A / Z, descending (numpy SVD), and the
    spectral norm of A~ A~^T - I, the quantity Sec. 4.2.2 argues is small."""
    A, Z = _f64(A), _f64(Z)
    R, Dr = d.merge_regions, A.shape[2]
    sv = np.empty((d.B, R, Dr), np.float64)
    dev = np.empty((d.B, R), np.float64)
    for b in range(d.B):
        for rho in range(R):
            z = np.maximum(Z[b, rho * Dr:(rho + 1) * Dr], 1e-20)
            At = A[b, rho] / z[:, None]
            sv[b, rho] = np.linalg.svd(At, compute_uv=False)
            dev[b, rho] = np.abs(np.linalg.eigvalsh(At @ At.T) - 1.0).max()
    return sv, dev


def layer(d, X, Wq, Wk, Wv, heads, Xe=None, Wo=None, idx=None, AZ=None):
    """Alg. 3 end to end.  idx / AZ given = pattern reuse (Sec. 4.3.2): a cached idx skips the
    selection, a cached (A, Z) also skips the weights; both are applied to the CURRENT X."""
    out = {}
    if AZ is None:
        if idx is None:
            idx, gain, gap = select(d, X)
            out["gain"], out["gap"] = gain, gap
        A, Z, clamps = merge_weights(d, X, idx)
        out["clamps"] = clamps
    else:
        A, Z = AZ
    Xm = merge(d, X, A, Z)
    O = attend(Xm, Xe, Wq, Wk, Wv, heads, Wo)
    Y = unmerge(d, A, Z, O)
    D = Xm.shape[1]
    out.update(idx=idx, A=A, Z=Z, Xm=Xm, O=O, Y=Y, Y_extra=O[:, D:, :])
    return out


def threads():
    """Number of OpenMP threads the oracle's parallel loops use on this host."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    return len(os.sched_getaffinity(0))
