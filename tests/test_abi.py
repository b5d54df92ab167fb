"""The C-ABI library loads and exports every symbol include/dyllm.h declares; host-side argument
checks work without a GPU (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

from paper_2603_08026_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "dyllm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dyllm_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2603_08026_amd import build
        build.build(verbose=False)
    return B.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.SYMBOLS) == names


def test_strerror_and_codes(lib):
    assert lib.dyllm_strerror(0) == b"ok"
    for code in range(-6, 0):
        assert lib.dyllm_strerror(code) not in (b"ok", b"unknown error")
    assert lib.dyllm_strerror(-99) == b"unknown error"


def _cfg(**kw):
    base = dict(hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=768, max_batch=1, max_seq=128,
                max_rows=0, dtype=B.F32, rms_eps=1e-5, rope_theta=10000.0)
    base.update(kw)
    return B.LayerCfg(**base)


def test_workspace_bytes_and_config_checks(lib):
    n = B.workspace_bytes(_cfg())
    assert n > 128 * 768 * 4
    assert B.workspace_bytes(_cfg(max_rows=16)) < n
    big = B.workspace_bytes(_cfg(hidden=4096, n_heads=32, n_kv_heads=32, head_dim=128, ffn_dim=12288,
                                 max_batch=16, max_seq=1280, dtype=B.BF16))
    assert 1 << 30 < big < 8 << 30
    for bad, code in [
        (_cfg(head_dim=48), -3), (_cfg(n_kv_heads=3), -2), (_cfg(hidden=100), -3), (_cfg(dtype=7), -1),
        (_cfg(max_seq=0), -1), (_cfg(max_rows=129), -2), (_cfg(dtype=B.BF16, hidden=192), -3),
    ]:
        with pytest.raises(B.DyllmError) as e:
            B.workspace_bytes(bad)
        assert e.value.code == code
    out = C.c_void_p()
    assert lib.dyllm_create(None, C.byref(out)) == -1
    assert lib.dyllm_create(C.byref(_cfg(head_dim=48)), C.byref(out)) == -3
    assert lib.dyllm_destroy(None) == -1
    assert lib.dyllm_full_step(None, None, None, None, 1, 1, None) == -1
    assert lib.dyllm_layer_step(None, None, None, None, None, 1, 1, 0.5, None, None, None) == -1


def test_cache_memory_ratio_matches_paper_formula():
    # K+V+C+OUT bytes per token over K+V only: (2d/g + 2d)/(2d/g)  [Sec. 5]
    for d, H, Hkv, dh, want in [(4096, 32, 32, 128, 2), (3584, 28, 4, 128, 8)]:
        kv = 2 * Hkv * dh
        assert (kv + H * dh + d) / kv == want
