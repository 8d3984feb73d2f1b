"""ctypes binding of libattnring.so: the same entry points as include/attnring.h.

Argument marshalling only.  Tensors are torch tensors on the GPU (torch is used
for device memory and streams, nothing else); every step of the computation
runs in the library's HIP kernels.  There is no CPU fallback: if the library is
not built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattnring.so")

ATTN_OK, ATTN_ERR_INVALID, ATTN_ERR_SHAPE, ATTN_ERR_UNSUPPORTED, ATTN_ERR_ALLOC, ATTN_ERR_DEVICE = range(6)
ATTN_SCHEME_FULL, ATTN_SCHEME_SYMMETRIC, ATTN_SCHEME_CAUSAL = 0, 1, 2
ATTN_F32, ATTN_BF16 = 0, 1
ATTN_FLAG_NO_SKIP = 1
ATTN_FLAG_WIDE_TILES = 2
ATTN_FLAG_NARROW_TILES = 4
ATTN_FLAG_SKIP_PADDED_ROWS = 8
ATTN_FLAG_FUSE_Q_PROJECTION = 16

EXPORTS = ("attn_init", "attn_set_key_lengths", "attn_forward", "attn_forward_packed", "attn_forward_static", "attn_stats",
           "attn_profile", "attn_profile_read", "attn_last_error", "attn_destroy")
ATTN_STATIC_SCRATCH_MIB = 64


class attn_config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_k", C.c_int32), ("p", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float),
                ("flags", C.c_uint32)]


class attn_stats_t(C.Structure):
    _fields_ = [("pairs_full", C.c_uint64), ("pairs_needed", C.c_uint64 * 3),
                ("pairs_scheduled", C.c_uint64 * 3), ("tiles_full", C.c_uint64),
                ("tiles_executed", C.c_uint64), ("pairs_executed", C.c_uint64),
                ("phys_tiles_executed", C.c_uint64), ("phys_br", C.c_int32), ("phys_bc", C.c_int32),
                ("proj_gemms", C.c_uint64)]


class attn_profile_t(C.Structure):
    _fields_ = [("calls", C.c_int32), ("ms_prepare", C.c_float), ("ms_projection", C.c_float),
                ("ms_attention", C.c_float)]


class AttnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"attnring status {status}: {text}")
        self.status = status


_lib = None


def load():
    """Load libattnring.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2012_01114_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    lib.attn_init.restype = C.c_int
    lib.attn_init.argtypes = [C.POINTER(attn_config), C.POINTER(vp)]
    lib.attn_set_key_lengths.restype = C.c_int
    lib.attn_set_key_lengths.argtypes = [vp, vp]
    lib.attn_forward.restype = C.c_int
    lib.attn_forward.argtypes = [vp, vp, vp, vp, vp, C.c_int32, vp, vp]
    lib.attn_forward_packed.restype = C.c_int
    lib.attn_forward_packed.argtypes = [vp, vp, vp, vp, vp, vp, C.c_int32, vp, vp]
    lib.attn_forward_static.restype = C.c_int
    lib.attn_forward_static.argtypes = [C.POINTER(attn_config), vp, vp, vp, vp, vp, C.c_int32, vp, vp]
    lib.attn_stats.restype = C.c_int
    lib.attn_stats.argtypes = [vp, C.POINTER(attn_stats_t)]
    lib.attn_profile.restype = C.c_int
    lib.attn_profile.argtypes = [vp, C.c_int32]
    lib.attn_profile_read.restype = C.c_int
    lib.attn_profile_read.argtypes = [vp, C.POINTER(attn_profile_t)]
    lib.attn_last_error.restype = C.c_char_p
    lib.attn_last_error.argtypes = [vp]
    lib.attn_destroy.restype = None
    lib.attn_destroy.argtypes = [vp]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("attnring takes contiguous GPU tensors")
    return t.data_ptr()


def _check(status: int, ctx) -> None:
    if status != ATTN_OK:
        raise AttnError(status, attn_last_error(ctx))


def attn_last_error(ctx) -> str:
    return load().attn_last_error(ctx).decode()


def attn_init(batch: int, n: int, d_model: int, n_heads: int, d_k: int, p: int, dtype: int,
              scale: float = 0.0, flags: int = 0):
    """Returns the opaque context handle (a c_void_p)."""
    cfg = attn_config(batch, n, d_model, n_heads, d_k, p, dtype, scale, flags)
    ctx = C.c_void_p()
    st = load().attn_init(C.byref(cfg), C.byref(ctx))
    _check(st, None)
    return ctx


def attn_set_key_lengths(ctx, lens_dev) -> None:
    """lens_dev: int32 GPU tensor [batch] or None; the caller keeps it alive."""
    if lens_dev is not None:
        import torch
        if lens_dev.dtype != torch.int32:
            raise ValueError("key lengths must be int32")
    _check(load().attn_set_key_lengths(ctx, _ptr(lens_dev)), ctx)


def attn_forward(ctx, X, Wq, Wk, Wv, scheme: int, out, stream=None) -> None:
    """Enqueue one forward pass on `stream` (a torch.cuda.Stream; default: the current one)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(X.device)
    st = load().attn_forward(ctx, _ptr(X), _ptr(Wq), _ptr(Wk), _ptr(Wv), int(scheme), _ptr(out),
                             C.c_void_p(stream.cuda_stream))
    _check(st, ctx)


def attn_forward_packed(ctx, row_offsets_dev, X, Wq, Wk, Wv, scheme: int, out, stream=None) -> None:
    """attn_forward on items stored back to back: item b is rows row_offsets_dev[b] .. row_offsets_dev[b+1]-1
    of X and out (row_offsets_dev: int32 GPU tensor of batch + 1 entries)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(X.device)
    st = load().attn_forward_packed(ctx, _ptr(row_offsets_dev), _ptr(X), _ptr(Wq), _ptr(Wk), _ptr(Wv), int(scheme),
                                    _ptr(out), C.c_void_p(stream.cuda_stream))
    _check(st, ctx)


def attn_forward_static(batch: int, n: int, d_model: int, n_heads: int, d_k: int, p: int, dtype: int,
                        X, Wq, Wk, Wv, scheme: int, out, lens_dev=None, scale: float = 0.0, flags: int = 0,
                        stream=None) -> None:
    """attn_forward on the library's fixed workspace: no context, no allocation."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(X.device)
    cfg = attn_config(batch, n, d_model, n_heads, d_k, p, dtype, scale, flags)
    st = load().attn_forward_static(C.byref(cfg), _ptr(lens_dev), _ptr(X), _ptr(Wq), _ptr(Wk), _ptr(Wv),
                                    int(scheme), _ptr(out), C.c_void_p(stream.cuda_stream))
    _check(st, None)


def attn_stats(ctx) -> dict:
    st = attn_stats_t()
    _check(load().attn_stats(ctx, C.byref(st)), ctx)
    return {"pairs_full": st.pairs_full, "pairs_needed": list(st.pairs_needed),
            "pairs_scheduled": list(st.pairs_scheduled), "tiles_full": st.tiles_full,
            "tiles_executed": st.tiles_executed, "pairs_executed": st.pairs_executed,
            "phys_tiles_executed": st.phys_tiles_executed, "phys_br": st.phys_br, "phys_bc": st.phys_bc,
            "proj_gemms": st.proj_gemms}


def attn_profile(ctx, enable: bool) -> None:
    _check(load().attn_profile(ctx, 1 if enable else 0), ctx)


def attn_profile_read(ctx) -> dict:
    pr = attn_profile_t()
    _check(load().attn_profile_read(ctx, C.byref(pr)), ctx)
    return {"calls": pr.calls, "ms_prepare": pr.ms_prepare, "ms_projection": pr.ms_projection,
            "ms_attention": pr.ms_attention}


def attn_destroy(ctx) -> None:
    load().attn_destroy(ctx)
