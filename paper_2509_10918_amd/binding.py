"""Thin ctypes binding of libtoma's C ABI (include/toma.h): same names, argument marshalling only.

Every function takes torch CUDA tensors (device memory and the current stream come from torch),
hands raw pointers to the library and raises TomaError on a non-zero status.  There is no CPU
path: if libtoma.so has not been built, loading it fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# (a process started with TOMA_SANITIZE=1 loads the host-sanitizer build instead: CPU argument checks only)
LIB_PATH = os.path.join(_HERE, "libtoma_san.so" if os.environ.get("TOMA_SANITIZE", "0") == "1" else "libtoma.so")

TOMA_F32, TOMA_BF16 = 0, 1
TOMA_REUSE_IDX, TOMA_REUSE_A, TOMA_RECOMPUTE_WEIGHTS = 1, 2, 4
EXPORTS = ("toma_workspace_bytes", "toma_status_string", "toma_select", "toma_select_static", "toma_merge", "toma_map_bytes",
           "toma_map_build", "toma_merge_cached", "toma_attend", "toma_cross_attend", "toma_unmerge", "toma_unmerge_pinv", "toma_recompute_cache_bytes", "toma_merge_recompute",
           "toma_unmerge_recompute", "toma_layer", "toma_mlp", "toma_profile_enable",
           "toma_profile_kernel_name", "toma_profile_read", "toma_profile_map_product", "toma_profile_greedy_parts")


class TomaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class toma_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32), ("C", ctypes.c_int32),
                ("tile_h", ctypes.c_int32), ("tile_w", ctypes.c_int32), ("d_loc", ctypes.c_int32),
                ("merge_regions", ctypes.c_int32), ("tau", ctypes.c_float), ("logit_scale", ctypes.c_float),
                ("dtype", ctypes.c_int32)]

    @property
    def P(self):
        return (self.H // self.tile_h) * (self.W // self.tile_w)

    @property
    def N(self):
        return self.H * self.W

    @property
    def D(self):
        return self.P * self.d_loc


class toma_attn_desc(ctypes.Structure):
    _fields_ = [("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("t_extra", ctypes.c_int32)]


_lib = None


def lib():
    """Load libtoma.so (built by `python -m paper_2509_10918_amd.build`); no fallback exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with paper_2509_10918_amd/build.py "
                              "(hipcc, gfx950); there is no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        L.toma_workspace_bytes.restype = ctypes.c_size_t
        L.toma_workspace_bytes.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        L.toma_status_string.restype = ctypes.c_char_p
        L.toma_status_string.argtypes = [ctypes.c_int]
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.toma_select.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
        L.toma_select_static.argtypes = [vp, vp, vp, vp, vp, vp]
        L.toma_select_static.restype = ctypes.c_int
        L.toma_merge.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.toma_map_bytes.restype = ctypes.c_size_t
        L.toma_map_bytes.argtypes = [vp]
        L.toma_map_build.argtypes = [vp, vp, vp, vp]
        L.toma_merge_cached.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.toma_attend.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.toma_cross_attend.argtypes = [vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.toma_cross_attend.restype = ctypes.c_int
        L.toma_unmerge.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp, sz, vp]
        L.toma_recompute_cache_bytes.restype = ctypes.c_size_t
        L.toma_recompute_cache_bytes.argtypes = [vp]
        L.toma_merge_recompute.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.toma_merge_recompute.restype = ctypes.c_int
        L.toma_unmerge_recompute.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp, sz, vp]
        L.toma_unmerge_recompute.restype = ctypes.c_int
        L.toma_unmerge_pinv.argtypes = [vp, vp, vp, vp, ctypes.c_int32, ctypes.c_float, vp, vp, sz, vp]
        L.toma_unmerge_pinv.restype = ctypes.c_int
        L.toma_layer.argtypes = [vp, vp, ctypes.c_uint32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.toma_mlp.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp]
        for name in ("toma_select", "toma_merge", "toma_map_build", "toma_merge_cached", "toma_attend", "toma_cross_attend", "toma_unmerge", "toma_unmerge_pinv", "toma_recompute_cache_bytes", "toma_merge_recompute",
           "toma_unmerge_recompute",
                     "toma_layer", "toma_mlp"):
            getattr(L, name).restype = ctypes.c_int
        L.toma_profile_enable.argtypes = [ctypes.c_int]
        L.toma_profile_kernel_name.restype = ctypes.c_char_p
        L.toma_profile_kernel_name.argtypes = [ctypes.c_int]
        L.toma_profile_read.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)]
        L.toma_profile_map_product.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_int32)]
        L.toma_profile_map_product.restype = ctypes.c_int
        L.toma_profile_greedy_parts.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.toma_profile_greedy_parts.restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status):
    return lib().toma_status_string(int(status)).decode()


def make_desc(B, H, W, C, tile_h, tile_w, d_loc, merge_regions, tau, dtype, logit_scale=0.0):
    code = {torch.float32: TOMA_F32, torch.bfloat16: TOMA_BF16, "f32": TOMA_F32, "bf16": TOMA_BF16}[dtype]
    return toma_desc(B, H, W, C, tile_h, tile_w, d_loc, merge_regions, tau, logit_scale, code)


def torch_dtype(desc):
    return torch.bfloat16 if desc.dtype == TOMA_BF16 else torch.float32


def _ref(s):
    return None if s is None else ctypes.addressof(s)


def _ptr(t):
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError("libtoma takes contiguous CUDA tensors")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(status, where):
    if status != 0:
        raise TomaError(status, where)


def toma_workspace_bytes(desc, attn=None):
    return lib().toma_workspace_bytes(_ref(desc), _ref(attn))


def alloc_workspace(desc, attn=None, device="cuda"):
    n = toma_workspace_bytes(desc, attn)
    if n == 0:
        raise TomaError(2, "toma_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def toma_select(desc, X, idx, gain, gap, ws):
    _check(lib().toma_select(_ref(desc), _ptr(X), _ptr(idx), _ptr(gain), _ptr(gap), _ptr(ws), ws.numel(),
                             _stream()), "toma_select")


def toma_select_static(desc, X, idx, gain, gap):
    _check(lib().toma_select_static(_ref(desc), _ptr(X), _ptr(idx), _ptr(gain), _ptr(gap), _stream()),
           "toma_select_static")


def toma_merge(desc, X, idx, A, Z, amap, Xm, ws):
    _check(lib().toma_merge(_ref(desc), _ptr(X), _ptr(idx), _ptr(A), _ptr(Z), _ptr(amap), _ptr(Xm), _ptr(ws),
                            ws.numel(), _stream()), "toma_merge")


def toma_map_bytes(desc):
    return lib().toma_map_bytes(_ref(desc))


def toma_map_build(desc, A, amap):
    _check(lib().toma_map_build(_ref(desc), _ptr(A), _ptr(amap), _stream()), "toma_map_build")


def toma_merge_cached(desc, X, A, Z, amap, Xm, ws):
    _check(lib().toma_merge_cached(_ref(desc), _ptr(X), _ptr(A), _ptr(Z), _ptr(amap), _ptr(Xm), _ptr(ws),
                                   ws.numel(), _stream()), "toma_merge_cached")


def toma_attend(desc, attn, Xm, X_extra, Wq, Wk, Wv, Wo, O, ws):
    _check(lib().toma_attend(_ref(desc), _ref(attn), _ptr(Xm), _ptr(X_extra), _ptr(Wq), _ptr(Wk), _ptr(Wv),
                             _ptr(Wo), _ptr(O), _ptr(ws), ws.numel(), _stream()), "toma_attend")


def toma_cross_attend(desc, attn, U, Ctx, Wq, Wk, Wv, Wo, O, ws):
    _check(lib().toma_cross_attend(_ref(desc), _ref(attn), _ptr(U), _ptr(Ctx), Ctx.shape[1], Ctx.shape[2], _ptr(Wq),
                                   _ptr(Wk), _ptr(Wv), _ptr(Wo), _ptr(O), _ptr(ws), ws.numel(), _stream()),
           "toma_cross_attend")


def toma_unmerge(desc, A, Z, amap, O, Y, ws):
    _check(lib().toma_unmerge(_ref(desc), _ptr(A), _ptr(Z), _ptr(amap), _ptr(O), O.shape[1], _ptr(Y), _ptr(ws),
                              ws.numel(), _stream()), "toma_unmerge")


def toma_recompute_cache_bytes(desc):
    return lib().toma_recompute_cache_bytes(_ref(desc))


def toma_merge_recompute(desc, X, idx, Z, wcache, Xm, ws):
    _check(lib().toma_merge_recompute(_ref(desc), _ptr(X), _ptr(idx), _ptr(Z), _ptr(wcache), _ptr(Xm), _ptr(ws),
                                      ws.numel(), _stream()), "toma_merge_recompute")


def toma_unmerge_recompute(desc, X, idx, Z, wcache, O, Y, ws):
    _check(lib().toma_unmerge_recompute(_ref(desc), _ptr(X), _ptr(idx), _ptr(Z), _ptr(wcache), _ptr(O), O.shape[1],
                                        _ptr(Y), _ptr(ws), ws.numel(), _stream()), "toma_unmerge_recompute")


def toma_unmerge_pinv(desc, A, Z, O, rcond, Y, ws):
    _check(lib().toma_unmerge_pinv(_ref(desc), _ptr(A), _ptr(Z), _ptr(O), O.shape[1], float(rcond), _ptr(Y), _ptr(ws),
                                   ws.numel(), _stream()), "toma_unmerge_pinv")


def toma_layer(desc, attn, reuse_flags, X, X_extra, idx, A, Z, amap, Wq, Wk, Wv, Wo, Y, Y_extra, ws):
    _check(lib().toma_layer(_ref(desc), _ref(attn), int(reuse_flags), _ptr(X), _ptr(X_extra), _ptr(idx), _ptr(A),
                            _ptr(Z), _ptr(amap), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(Wo), _ptr(Y), _ptr(Y_extra),
                            _ptr(ws), ws.numel(), _stream()), "toma_layer")


def toma_mlp(In, W1, W2, Hbuf, Out):
    """Out = gelu(In W1) W2 on the rows of In ([..., C]); Hbuf is [rows, hidden] scratch."""
    C, hidden = W1.shape
    rows = In.numel() // C
    code = TOMA_BF16 if In.dtype == torch.bfloat16 else TOMA_F32
    _check(lib().toma_mlp(code, rows, C, hidden, _ptr(In), _ptr(W1), _ptr(W2), _ptr(Hbuf), _ptr(Out), _stream()),
           "toma_mlp")


def toma_profile_enable(on):
    _check(lib().toma_profile_enable(1 if on else 0), "toma_profile_enable")


def toma_profile_kernel_names():
    names, i = [], 0
    while True:
        n = lib().toma_profile_kernel_name(i)
        if n is None:
            return names
        names.append(n.decode())
        i += 1


def toma_profile_read(kernel):
    """(launches, total milliseconds) of one kernel since the last read; clears them."""
    n, ms = ctypes.c_int32(0), ctypes.c_float(0.0)
    _check(lib().toma_profile_read(kernel.encode(), ctypes.byref(n), ctypes.byref(ms)), "toma_profile_read")
    return n.value, ms.value


def toma_profile_map_product(desc, which):
    """(rows, columns, K split) of the block tile of the merge (0) / unmerge (1) product or of the write
    pass of the two-pass weights (2), or None."""
    out = (ctypes.c_int32 * 3)()
    rc = lib().toma_profile_map_product(_ref(desc), int(which), out)
    return None if rc != 0 else tuple(out)


def toma_profile_greedy_parts(desc, X, idx, parts, ws):
    """toma_select through the greedy kernel that times the parts of its rounds; parts: int64
    [B * P, waves, 8] (waves = 8 for regions of 256 tokens, 2 for regions of 64)."""
    _check(lib().toma_profile_greedy_parts(_ref(desc), _ptr(X), _ptr(idx), _ptr(parts), _ptr(ws), ws.numel(), _stream()),
           "toma_profile_greedy_parts")


def alloc_cache(desc, device="cuda"):
    """Caller-owned pattern cache (idx, A, Z, amap) of one layer; amap is None when the shape uses no
    block map."""
    dt = torch_dtype(desc)
    R = desc.merge_regions
    idx = torch.empty((desc.B, desc.P, desc.d_loc), dtype=torch.int32, device=device)
    A = torch.empty((desc.B, R, desc.D // R, desc.N // R), dtype=dt, device=device)
    Z = torch.empty((desc.B, desc.D), dtype=torch.float32, device=device)
    n = toma_map_bytes(desc)
    amap = torch.empty(n, dtype=torch.uint8, device=device) if n else None
    return idx, A, Z, amap
