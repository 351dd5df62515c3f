"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/qjl.h declares, and rejects bad arguments on the host
before anything is launched (no compute call is made here)."""
import ctypes
import os
import re

import pytest

import paper_2406_03482_amd as qjl
from paper_2406_03482_amd import QJLShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, INVALID, UNSUPPORTED, WORKSPACE, HIP = 0, -1, -2, -3, -4


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(qjl.lib_path()):
        from paper_2406_03482_amd import build
        build.build(verbose=False)
    return qjl.lib()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "qjl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qjl_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    names = _declared_symbols()
    assert names == ["qjl_append_keys", "qjl_decode_attention", "qjl_decode_attention_dual",
                     "qjl_decode_attention_dual_vq", "qjl_decode_attention_noalloc", "qjl_decode_attention_splits", "qjl_decode_attention_timed",
                     "qjl_decode_attention_vq", "qjl_decode_dual_workspace_bytes", "qjl_decode_noalloc_max_bytes", "qjl_decode_plan", "qjl_decode_step",
                     "qjl_decode_workspace_bytes", "qjl_generation_step", "qjl_generation_step_devpos",
                     "qjl_make_dual_sketch", "qjl_make_sketch", "qjl_make_sketch_orthogonal", "qjl_outlier_workspace_bytes",
                     "qjl_project_query", "qjl_quantize_keys", "qjl_quantize_keys_dual", "qjl_quantize_values",
                     "qjl_scores", "qjl_select_outliers", "qjl_status_string", "qjl_version"]
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_strings(L):
    assert L.qjl_version() >= 100
    texts = {s: L.qjl_status_string(s).decode() for s in (OK, INVALID, UNSUPPORTED, WORKSPACE, HIP, -99)}
    assert texts[OK] == "ok" and len(set(texts.values())) == 6


def test_struct_layout_matches_header():
    assert ctypes.sizeof(QJLShape) == 32
    assert [f[0] for f in QJLShape._fields_] == ["batch", "q_heads", "kv_heads", "n", "d", "m",
                                                 "dtype", "scale"]


GOOD = dict(batch=1, q_heads=32, kv_heads=8, n=4096, d=128, m=256, dtype=2, scale=1.0)
PTR = 0x1000  # never dereferenced: every call below must fail validation first


def _sh(**kw):
    a = dict(GOOD)
    a.update(kw)
    return QJLShape(a["batch"], a["q_heads"], a["kv_heads"], a["n"], a["d"], a["m"], a["dtype"], a["scale"])


def test_null_and_misaligned_pointers_are_rejected(L):
    sh = _sh()
    assert L.qjl_make_sketch(1, 256, 128, 2, None, None) == INVALID
    assert L.qjl_make_sketch(1, 256, 128, 2, PTR + 2, None) == INVALID
    assert L.qjl_make_sketch(1, 0, 128, 2, PTR, None) == INVALID
    assert L.qjl_make_sketch(1, 256, 128, 7, PTR, None) == INVALID
    assert L.qjl_quantize_keys(None, PTR, PTR, PTR, PTR, None) == INVALID
    for bad in range(4):
        args = [PTR] * 4
        args[bad] = None
        assert L.qjl_quantize_keys(ctypes.byref(sh), *args, None) == INVALID
        args[bad] = PTR + 4
        assert L.qjl_quantize_keys(ctypes.byref(sh), *args, None) == INVALID
    for bad in range(3):
        args = [PTR] * 3
        args[bad] = None
        assert L.qjl_project_query(ctypes.byref(sh), *args, None) == INVALID
    for bad in range(4):
        args = [PTR] * 4
        args[bad] = None
        assert L.qjl_scores(ctypes.byref(sh), *args, None) == INVALID
    for bad in range(6):
        args = [PTR] * 6
        args[bad] = None
        assert L.qjl_decode_attention(ctypes.byref(sh), *args, PTR, 1 << 30, None) == INVALID


@pytest.mark.parametrize("field,value", [("batch", 0), ("q_heads", 0), ("kv_heads", 0), ("n", 0),
                                         ("n", -5), ("d", 0), ("m", 0), ("dtype", 3), ("dtype", -1),
                                         ("kv_heads", 5), ("scale", float("nan"))])
def test_invalid_shapes_are_rejected(L, field, value):
    sh = _sh(**{field: value})
    assert L.qjl_quantize_keys(ctypes.byref(sh), PTR, PTR, PTR, PTR, None) == INVALID
    assert L.qjl_project_query(ctypes.byref(sh), PTR, PTR, PTR, None) == INVALID
    assert L.qjl_scores(ctypes.byref(sh), PTR, PTR, PTR, PTR, None) == INVALID
    assert L.qjl_decode_attention(ctypes.byref(sh), PTR, PTR, PTR, PTR, PTR, PTR, PTR, 1 << 30, None) == INVALID
    assert L.qjl_decode_workspace_bytes(ctypes.byref(sh)) == 0


def test_unsupported_shapes_are_reported_as_such(L):
    assert L.qjl_quantize_keys(ctypes.byref(_sh(m=100)), PTR, PTR, PTR, PTR, None) == UNSUPPORTED
    assert L.qjl_quantize_keys(ctypes.byref(_sh(d=4096)), PTR, PTR, PTR, PTR, None) == UNSUPPORTED
    assert L.qjl_scores(ctypes.byref(_sh(m=96)), PTR, PTR, PTR, PTR, None) == UNSUPPORTED
    for kw in (dict(d=64), dict(m=96), dict(m=1024)):
        sh = _sh(**kw)
        assert L.qjl_decode_workspace_bytes(ctypes.byref(sh)) == 0
        assert L.qjl_decode_attention(ctypes.byref(sh), PTR, PTR, PTR, PTR, PTR, PTR, PTR, 1 << 30,
                                      None) == UNSUPPORTED


def test_workspace_contract(L):
    sh = _sh()
    need = L.qjl_decode_workspace_bytes(ctypes.byref(sh))
    assert need > 0 and need % 256 == 0
    # room for S q alone is a lower bound
    assert need >= GOOD["batch"] * GOOD["q_heads"] * GOOD["m"] * 4
    call = lambda ws, nbytes: L.qjl_decode_attention(ctypes.byref(sh), PTR, PTR, PTR, PTR, PTR, PTR,
                                                     ws, nbytes, None)
    assert call(None, need) == WORKSPACE
    assert call(0x10000, need - 1) == WORKSPACE
    assert call(0x10000 + 16, need) == INVALID          # workspace must be 256-byte aligned
    # grows with the problem, never shrinks below the S q area
    big = L.qjl_decode_workspace_bytes(ctypes.byref(_sh(batch=16)))
    assert big > need


def test_python_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        qjl.qjl_project_query(torch.zeros(1, 1, 128), torch.zeros(256, 128))


def test_dual_entry_points_validate_on_the_host(L):
    """Outlier-channel calls: bad arguments are turned into status codes before any launch."""
    sh = QJLShape(1, 4, 2, 100, 128, 256, 2, 1.0)
    ok = ctypes.c_void_p(0x1000)                     # aligned, never dereferenced: every call below fails earlier
    vp = ctypes.c_void_p
    L.qjl_outlier_workspace_bytes.restype = ctypes.c_size_t
    L.qjl_decode_dual_workspace_bytes.restype = ctypes.c_size_t
    assert L.qjl_outlier_workspace_bytes(ctypes.byref(sh)) == 1 * 2 * 1 * 128 * 4
    assert L.qjl_decode_dual_workspace_bytes(ctypes.byref(sh), 128) > 0
    assert L.qjl_decode_dual_workspace_bytes(ctypes.byref(sh), 64) == 0       # unsupported split
    big = QJLShape(1, 4, 2, 100, 128, 512, 2, 1.0)
    assert L.qjl_decode_dual_workspace_bytes(ctypes.byref(big), 128) > 0       # 512 + 128 bits: built
    assert L.qjl_decode_dual_workspace_bytes(ctypes.byref(big), 256) == 0      # 512 + 256: not
    bad = QJLShape(1, 4, 2, 100, 128, 384, 2, 1.0)
    assert L.qjl_decode_dual_workspace_bytes(ctypes.byref(bad), 128) == 0
    # count out of range / null pointers
    assert L.qjl_select_outliers(ctypes.byref(sh), ok, 0, ok, ok, ctypes.c_size_t(1 << 20), None) == INVALID
    assert L.qjl_select_outliers(ctypes.byref(sh), ok, 17, ok, ok, ctypes.c_size_t(1 << 20), None) == INVALID
    assert L.qjl_select_outliers(ctypes.byref(sh), ok, 4, ok, ok, ctypes.c_size_t(16), None) == WORKSPACE
    assert L.qjl_select_outliers(ctypes.byref(sh), vp(None), 4, ok, ok, ctypes.c_size_t(1 << 20), None) == INVALID
    assert L.qjl_make_dual_sketch(ctypes.byref(sh), 0, ok, ok, ok, 4, ok, None) == INVALID
    assert L.qjl_make_dual_sketch(ctypes.byref(sh), 128, ok, vp(None), ok, 4, ok, None) == INVALID
    assert L.qjl_quantize_keys_dual(ctypes.byref(sh), 128, ok, ok, vp(None), 4, ok, ok, ok, None) == INVALID
    odd = QJLShape(1, 4, 2, 100, 128, 250, 2, 1.0)
    assert L.qjl_quantize_keys_dual(ctypes.byref(odd), 128, ok, ok, ok, 4, ok, ok, ok, None) == UNSUPPORTED
    assert L.qjl_decode_attention_dual(ctypes.byref(sh), 128, ok, ok, ok, ok, ok, ok, ok, vp(None),
                                       ctypes.c_size_t(0), None, None, None) == WORKSPACE
    assert L.qjl_decode_attention_dual(ctypes.byref(sh), 64, ok, ok, ok, ok, ok, ok, ok, ok,
                                       ctypes.c_size_t(1 << 30), None, None, None) == UNSUPPORTED


def test_value_cache_entry_points_validate_on_the_host(L):
    sh = QJLShape(1, 4, 2, 100, 128, 256, 2, 1.0)
    ok = ctypes.c_void_p(0x1000)
    vp = ctypes.c_void_p
    assert L.qjl_quantize_values(ctypes.byref(sh), 4, vp(None), ok, ok, ok, None) == INVALID
    assert L.qjl_quantize_values(ctypes.byref(sh), 0, ok, ok, ok, ok, None) == INVALID
    assert L.qjl_quantize_values(ctypes.byref(sh), 3, ok, ok, ok, ok, None) == UNSUPPORTED      # codes of 2, 4 or 8 bits
    d64 = QJLShape(1, 4, 2, 100, 64, 256, 2, 1.0)
    assert L.qjl_quantize_values(ctypes.byref(d64), 4, ok, ok, ok, ok, None) == UNSUPPORTED
    args = (ok, ok, ok, ok, ok, ok, ok, ok)
    assert L.qjl_decode_attention_vq(ctypes.byref(sh), 4, *args, vp(None), ctypes.c_size_t(0), None, None, None) == WORKSPACE
    assert L.qjl_decode_attention_vq(ctypes.byref(sh), 3, *args, ok, ctypes.c_size_t(1 << 30), None, None, None) == UNSUPPORTED
    f32 = QJLShape(1, 4, 2, 100, 128, 256, 0, 1.0)
    assert L.qjl_decode_attention_vq(ctypes.byref(f32), 4, *args, ok, ctypes.c_size_t(1 << 30), None, None, None) == UNSUPPORTED
    assert L.qjl_decode_attention_vq(ctypes.byref(sh), 4, ok, ok, ok, ok, vp(None), ok, ok, ok, ok,
                                     ctypes.c_size_t(1 << 30), None, None, None) == INVALID


def test_orthogonal_sketch_entry_point_validates_on_the_host(L):
    ok = ctypes.c_void_p(0x1000)
    L.qjl_make_sketch_orthogonal.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_void_p, ctypes.c_void_p]
    assert L.qjl_make_sketch_orthogonal(1, 0, 128, 2, ok, None) == INVALID
    assert L.qjl_make_sketch_orthogonal(1, 256, 128, 7, ok, None) == INVALID
    assert L.qjl_make_sketch_orthogonal(1, 256, 128, 2, None, None) == INVALID
    assert L.qjl_make_sketch_orthogonal(1, 256, 256, 2, ok, None) == UNSUPPORTED      # a block must fit in LDS


def test_streaming_entry_points_validate_on_the_host(L):
    sh = QJLShape(1, 4, 2, 100, 128, 256, 2, 1.0)
    ok = ctypes.c_void_p(0x1000)
    assert L.qjl_append_keys(ctypes.byref(sh), -1, 1, ok, ok, ok, ok, None) == INVALID
    assert L.qjl_append_keys(ctypes.byref(sh), 99, 2, ok, ok, ok, ok, None) == INVALID        # past the capacity
    assert L.qjl_append_keys(ctypes.byref(sh), 0, 0, ok, ok, ok, ok, None) == INVALID
    assert L.qjl_append_keys(ctypes.byref(sh), 0, 1, None, ok, ok, ok, None) == INVALID
    d64 = QJLShape(1, 4, 2, 100, 64, 256, 2, 1.0)
    assert L.qjl_append_keys(ctypes.byref(d64), 0, 1, ok, ok, ok, ok, None) == UNSUPPORTED
    assert L.qjl_decode_step(ctypes.byref(sh), 100, ok, ok, ok, ok, ok, ok, ok, ok, ctypes.c_size_t(1 << 30), None) == INVALID
    assert L.qjl_decode_step(ctypes.byref(sh), 5, ok, ok, ok, ok, ok, ok, ok, None, ctypes.c_size_t(0), None) == WORKSPACE


# ------------------------------------------------------------------ the decode plan (host arithmetic only)
def _plan(L, splits=0, m_out=0, **kw):
    sh = _sh(**kw)
    out = (ctypes.c_int32 * 3)()
    L.qjl_decode_plan.restype = ctypes.c_size_t
    total = L.qjl_decode_plan(ctypes.byref(sh), m_out, splits, out)
    return int(total), int(out[0]), int(out[1]), int(out[2])


def test_forced_split_count_is_clamped_to_what_the_merge_kernel_holds(L):
    """The merge kernel keeps 512 chunk records' heads in LDS: no request may plan more."""
    for splits in (513, 1000, 4096, 2 ** 30):
        total, gt, nsplit, chunk = _plan(L, splits=splits, batch=1, q_heads=32, kv_heads=32, n=131072)
        assert 1 <= nsplit <= 512 and chunk % 64 == 0 and nsplit * chunk >= 131072
        assert total >= 1 * 32 * nsplit * 132 * 4
    # and never fewer than one 64-key block per wave
    total, gt, nsplit, chunk = _plan(L, splits=4096, batch=1, q_heads=8, kv_heads=2, n=5000)
    assert gt == 4 and nsplit == 10 and chunk == 512
    assert _plan(L, splits=-1)[0] == 0


@pytest.mark.parametrize("kw", [dict(batch=1, q_heads=32, kv_heads=8, n=33000), dict(batch=1, q_heads=1, kv_heads=1, n=70000),
                                dict(batch=2, q_heads=32, kv_heads=32, n=9999), dict(batch=1, q_heads=6, kv_heads=2, n=20011)])
def test_workspace_of_the_capacity_covers_every_shorter_context(L, kw):
    """A streaming generation sizes its workspace once, at the capacity of its caches (qjl_decode_step):
    the bytes of the plan must never decrease as the context grows, and every plan's records must fit its bytes."""
    cap = kw["n"]
    last = 0
    for n in list(range(1, 2050)) + list(range(2050, cap, 97)) + [cap]:
        total, gt, nsplit, chunk = _plan(L, **dict(kw, n=n))
        assert total >= last, (n, total, last)
        assert total >= kw["batch"] * kw["q_heads"] * nsplit * 132 * 4
        assert (nsplit - 1) * chunk < n <= nsplit * chunk
        last = total
    assert last == _plan(L, **kw)[0]
    L.qjl_decode_workspace_bytes.restype = ctypes.c_size_t
    assert L.qjl_decode_workspace_bytes(ctypes.byref(_sh(**kw))) == last
