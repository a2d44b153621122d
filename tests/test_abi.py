"""The C-ABI library: loads without a GPU, exports every symbol include/tdk.h declares, and rejects
bad arguments on the host before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2604_03143_amd import tdk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tdk.LIB_PATH):
        from paper_2604_03143_amd import _build
        _build.build(force=True)
    return tdk.load()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "tdk.h")).read() + open(os.path.join(ROOT, "include", "tdk_bench.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(tdk_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(tdk.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    assert tdk.tdk_status_str(tdk.OK) == "ok"
    assert "invalid" in tdk.tdk_status_str(tdk.ERR_INVALID_ARG)
    assert "gfx950" in tdk.tdk_version()
    assert tdk.tdk_kernel_name(tdk.KERNEL_FLAG) == "tdk_flag_kernel"


def _create(mdl, spans=(32,), pos0=(0,), sess=(0,), hist=(5,), tables=None):
    if tables is None:
        tables = [np.arange(8, dtype=np.int32) for _ in sess]
    return tdk.tdk_round_create(mdl, spans, pos0, sess, hist, tables)


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=64), tdk.ERR_UNSUPPORTED),
    (dict(page_tokens=8), tdk.ERR_UNSUPPORTED),
    (dict(num_kv_heads=16), tdk.ERR_UNSUPPORTED),
    (dict(dtype=3), tdk.ERR_UNSUPPORTED),
    (dict(rope_theta=0.0), tdk.ERR_INVALID_ARG),
    (dict(rope_theta=float("nan")), tdk.ERR_INVALID_ARG),
    (dict(rope_style=7), tdk.ERR_INVALID_ARG),
    (dict(num_layers=0), tdk.ERR_INVALID_ARG),
])
def test_create_rejects_bad_model(lib, kw, status):
    args = dict(num_layers=1)
    args.update(kw)
    with pytest.raises(tdk.TdkError) as e:
        _create(tdk.model(**args))
    assert e.value.status == status and e.value.detail


def test_create_rejects_bad_round(lib):
    m = tdk.model(1)
    with pytest.raises(tdk.TdkError) as e:
        _create(m, sess=(1,))
    assert e.value.status == tdk.ERR_INVALID_ARG and "session" in e.value.detail
    with pytest.raises(tdk.TdkError) as e:
        _create(m, hist=(-1,))
    assert e.value.status == tdk.ERR_INVALID_ARG
    with pytest.raises(tdk.TdkError) as e:
        _create(m, spans=(-1,))
    assert e.value.status == tdk.ERR_INVALID_ARG
    with pytest.raises(tdk.TdkError) as e:       # 5 + 32 tokens need 3 pages of 16
        _create(m, tables=[np.arange(2, dtype=np.int32)])
    assert e.value.status == tdk.ERR_INVALID_ARG and "too short" in e.value.detail
    with pytest.raises(tdk.TdkError) as e:
        _create(m, tables=[np.array([0, -1, 2], dtype=np.int32)])
    assert e.value.status == tdk.ERR_INVALID_ARG and "negative page" in e.value.detail
    with pytest.raises(tdk.TdkError) as e:
        _create(m, hist=(2 ** 31,), tables=[np.zeros(1, np.int32)])
    assert e.value.status == tdk.ERR_INVALID_ARG


def test_null_round_and_null_out(lib):
    io = tdk.layer_io(None, None, None, None, 0)
    assert lib.tdk_rerotate_round(None, 0, C.byref(io), None) == tdk.ERR_INVALID_ARG
    d = tdk.diff(None, None, None, None, 0, None)
    assert lib.tdk_diff_encode(None, 0, C.byref(io), C.c_float(0.01), C.byref(d), None) == tdk.ERR_INVALID_ARG
    assert lib.tdk_diff_decode(None, 0, C.byref(io), C.byref(d), None) == tdk.ERR_INVALID_ARG
    assert lib.tdk_round_create(None, None, 0, None, 0, None) == tdk.ERR_INVALID_ARG
    lib.tdk_round_destroy(None)
    assert lib.tdk_scratch_bytes(None) == 0
    assert lib.tdk_round_tune(None, 0, 0) == tdk.ERR_INVALID_ARG
    assert lib.tdk_util_copy(None, None, 16, None) == tdk.ERR_INVALID_ARG
    assert lib.tdk_util_fill(C.c_void_p(16), 0, 8, None) == tdk.ERR_INVALID_ARG


def test_storage_arithmetic_matches_printed_values(lib):
    """Sec. 6.4: 1 + (N-1)/R full caches; N = 10 -> about 1.8 (R = 11.2) and 1.5 (R = 17.5)."""
    assert abs(tdk.tdk_family_cost(10, 11.2) - 1.8) < 0.05
    assert abs(tdk.tdk_family_cost(10, 17.5) - 1.5) < 0.05
    m = tdk.model(48)
    assert tdk.tdk_dense_bytes(m, 5000) == 5000 * 4096
    assert tdk.tdk_diff_bytes(m, 19) == 19 * 65536 + 19 * 4 + 12


def test_product_does_not_import_oracle():
    """The product path never routes through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2604_03143_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
                assert "libtdo" not in src and "tdo_" not in src and "tdo.h" not in src, f
