"""C-ABI checks that need no GPU: the library loads, exports every function the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2012_01114_amd import attnring as ar

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "attnring.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = _declared()
    for must in ("attn_init", "attn_forward", "attn_stats"):
        assert must in names
    assert sorted(names) == sorted(ar.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = ar.load()
    for name in _declared():
        assert getattr(lib, name) is not None


def test_struct_layout_matches_header():
    assert C.sizeof(ar.attn_config) == 36
    assert C.sizeof(ar.attn_stats_t) == 11 * 8 + 2 * 4 + 8  # 11 u64, 2 i32, 1 u64
    assert C.sizeof(ar.attn_profile_t) == 16


def _init(**kw):
    cfg = dict(batch=1, n=16, d_model=64, n_heads=1, d_k=64, p=4, dtype=ar.ATTN_F32, scale=0.0, flags=0)
    cfg.update(kw)
    return ar.attn_init(**cfg)


@pytest.mark.parametrize("kw,status", [
    (dict(n=0), ar.ATTN_ERR_INVALID),
    (dict(batch=-1), ar.ATTN_ERR_INVALID),
    (dict(dtype=7), ar.ATTN_ERR_INVALID),
    (dict(flags=32), ar.ATTN_ERR_INVALID),
    (dict(flags=6), ar.ATTN_ERR_INVALID),
    (dict(scale=float("nan")), ar.ATTN_ERR_INVALID),
    (dict(n=18, p=4), ar.ATTN_ERR_SHAPE),          # n must be divisible by the ring partitions
    (dict(batch=4096, n=65536, n_heads=64, p=1), ar.ATTN_ERR_SHAPE),
    (dict(d_k=512), ar.ATTN_ERR_UNSUPPORTED),
])
def test_init_rejects_bad_config(kw, status):
    with pytest.raises(ar.AttnError) as e:
        _init(**kw)
    assert e.value.status == status
    assert len(str(e.value)) > 20


def test_null_arguments():
    lib = ar.load()
    assert lib.attn_init(None, None) == ar.ATTN_ERR_INVALID
    assert lib.attn_forward(None, None, None, None, None, 0, None, None) == ar.ATTN_ERR_INVALID
    assert lib.attn_stats(None, None) == ar.ATTN_ERR_INVALID
    assert lib.attn_profile(None, 1) == ar.ATTN_ERR_INVALID
    assert lib.attn_profile_read(None, None) == ar.ATTN_ERR_INVALID
    assert lib.attn_set_key_lengths(None, None) == ar.ATTN_ERR_INVALID
    assert lib.attn_forward_packed(None, None, None, None, None, None, 0, None, None) == ar.ATTN_ERR_INVALID
    assert lib.attn_forward_static(None, None, None, None, None, None, 0, None, None) == ar.ATTN_ERR_INVALID
    lib.attn_destroy(None)
    assert isinstance(ar.attn_last_error(None), str)


def test_static_entry_point_rejects_before_touching_the_device():
    """Shapes outside the matrix-core path and workspaces beyond the fixed array come back as
    UNSUPPORTED from the argument checks alone (the pointers are never followed)."""
    lib = ar.load()
    fake = C.c_void_p(0x10000)

    def call(**kw):
        cfg = dict(batch=1, n=512, d_model=128, n_heads=2, d_k=64, p=64, dtype=ar.ATTN_BF16, scale=0.0, flags=0)
        cfg.update(kw)
        c = ar.attn_config(*[cfg[k] for k in ("batch", "n", "d_model", "n_heads", "d_k", "p", "dtype", "scale", "flags")])
        return lib.attn_forward_static(C.byref(c), None, fake, fake, fake, fake, ar.ATTN_SCHEME_CAUSAL, fake, None)

    assert call(dtype=ar.ATTN_F32) == ar.ATTN_ERR_UNSUPPORTED
    assert call(d_k=32) == ar.ATTN_ERR_UNSUPPORTED
    assert call(d_model=72) == ar.ATTN_ERR_UNSUPPORTED
    assert call(n=18, p=4) == ar.ATTN_ERR_SHAPE
    assert call(batch=64, n=8192, n_heads=16) == ar.ATTN_ERR_UNSUPPORTED      # 3 x 1 GiB of q, k, v
    assert "bytes of workspace" in ar.attn_last_error(None)


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: no collectives, no sharding in this library."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
