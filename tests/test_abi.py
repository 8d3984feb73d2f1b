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
    (dict(flags=16), ar.ATTN_ERR_INVALID),
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
    lib.attn_destroy(None)
    assert isinstance(ar.attn_last_error(None), str)
