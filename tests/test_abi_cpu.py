"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, validates arguments before touching the device,
and reports a consistent parameter layout."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2109_15082_amd", "libmrem.so")


@pytest.fixture(scope="module")
def B():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    from paper_2109_15082_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "mrem.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(mrem_[a-z_0-9]+)\s*\(", header))
    assert len(declared) >= 14
    lib = ctypes.CDLL(LIB)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)


def test_config_validation(B):
    good = dict(n_layers=2, hidden=64, n_heads=2, ffn=256, max_batch=4, max_seq=32)
    ctx = B.mrem_create(**good)
    assert ctx
    B.mrem_destroy(ctx)
    for bad, status in [(dict(n_layers=0), B.MREM_ESHAPE), (dict(hidden=60), B.MREM_ESHAPE), (dict(n_heads=3), B.MREM_ESHAPE),
                        (dict(max_seq=1024), B.MREM_ESHAPE), (dict(w_bits=1), B.MREM_EINVAL), (dict(a_bits=9), B.MREM_EINVAL),
                        (dict(act_dtype=7), B.MREM_EINVAL), (dict(hidden=4096, n_heads=32), B.MREM_ESHAPE)]:
        with pytest.raises(B.MremError) as e:
            B.mrem_create(**{**good, **bad})
        assert e.value.status == status, bad
        assert str(e.value)


def test_parameter_layout(B):
    H, F, L = 64, 256, 3
    ctx = B.mrem_create(n_layers=L, hidden=H, n_heads=2, ffn=F, max_batch=4, max_seq=32)
    sizes = {"w_qkv": 3 * H * H, "w_o": H * H, "w_1": F * H, "w_2": H * F, "b_qkv": 3 * H, "b_o": H, "ln1_g": H, "ln1_b": H,
             "b_1": F, "b_2": H, "ln2_g": H, "ln2_b": H, "sw_qkv": 3 * H, "sw_o": H, "sw_1": F, "sw_2": H, "s_a": 8, "z_a": 8}
    per_layer = sum(sizes.values())
    assert B.mrem_param_count(ctx) == L * per_layer == B.mrem_teacher_count(ctx)
    for l in range(L):
        off = l * per_layer
        for name in B.FIELDS:
            assert B.mrem_param_size(ctx, name) == sizes[name]
            assert B.mrem_param_offset(ctx, l, name) == off
            assert off % 4 == 0                               # 16-byte aligned fields
            off += sizes[name]
    assert B.mrem_param_offset(ctx, L, "w_qkv") == -1 and B.mrem_param_offset(ctx, 0, 99) == -1
    assert B.mrem_teacher_cache_bytes(ctx) == 2 * L * (sizes["w_qkv"] + sizes["w_o"] + sizes["w_1"] + sizes["w_2"])
    w1, w2 = B.mrem_workspace_bytes(ctx, 2, 16), B.mrem_workspace_bytes(ctx, 4, 32)
    assert 0 < w1 < w2 and B.mrem_workspace_bytes(ctx, 0, 16) == 0
    B.mrem_destroy(ctx)


def test_entry_points_reject_bad_arguments_on_the_host(B):
    """Null pointers, sizes beyond the configured maxima and a short workspace are
    refused before any kernel is enqueued (so this runs without a GPU)."""
    lib = ctypes.CDLL(LIB)
    ctx = B.mrem_create(n_layers=1, hidden=64, n_heads=2, ffn=256, max_batch=4, max_seq=32)
    fake = ctypes.c_void_p(0x1000)      # aligned, never dereferenced on the host
    lib.mrem_module_step.restype = ctypes.c_int
    args = lambda ws, nbytes, batch=4, seq=32, params=fake, lam=0.0: B._lib.mrem_module_step(
        ctx, params, fake, fake, 1, 1e-3, lam, fake, fake, fake, fake, None, batch, seq, fake, fake, fake, None, ws, nbytes, None)
    need = B.mrem_workspace_bytes(ctx, 4, 32)
    assert args(fake, need - 1) == B.MREM_EWORKSPACE and "workspace" in B.mrem_last_error(ctx)
    assert args(None, need) == B.MREM_EINVAL
    assert args(fake, need, batch=5) == B.MREM_ESHAPE
    assert args(fake, need, seq=33) == B.MREM_ESHAPE
    assert args(fake, need, params=None) == B.MREM_EINVAL
    assert args(fake, need, params=ctypes.c_void_p(0x1004)) == B.MREM_EINVAL
    assert args(fake, need, lam=1.5) == B.MREM_EINVAL and "lambda" in B.mrem_last_error(ctx)
    assert B._lib.mrem_quantize(None, 4, 8, 4, 1, 1, fake, fake, None) == B.MREM_EINVAL
    assert B._lib.mrem_quantize(fake, 4, 8, 1, 1, 1, fake, fake, None) == B.MREM_EINVAL
    assert B._lib.mrem_quantize(fake, 4, 8, 4, 3, 1, fake, fake, None) == B.MREM_EINVAL
    # no flag given: the check says so; a misaligned flag is refused
    assert B._lib.mrem_check_nonfinite(ctx, None) == B.MREM_EINVAL
    assert B._lib.mrem_set_nonfinite_flag(ctx, ctypes.c_void_p(0x1002)) == B.MREM_EINVAL
    B.mrem_destroy(ctx)


def test_schedules_and_queue_bookkeeping_on_the_host(B):
    """Section 5.1.2 / 4.2.1 schedules against their formulas, and the ring of Algorithm 1's input queue:
    depth + 1 slots, first in first out, ages counted from the newest published entry (addresses only:
    nothing is dereferenced, so this runs without a GPU)."""
    import numpy as np
    for t in range(0, 11):
        assert B.mrem_schedule_lr(1e-4, t, 10) == 1e-4 * (1 - t / 10)
        assert B.mrem_schedule_lambda(t, 4) == max(1 - t / 4, 0)
    assert B.mrem_schedule_lambda(3, 0) == 0.0 and B.mrem_schedule_lr(1e-4, 0, 0) == 0.0
    half, lens, depth = 1000, 12, 3
    slot = 2 * 1024 + 256                                   # halves and lengths rounded up to 256 bytes
    assert B.mrem_queue_bytes(depth, half, lens) == (depth + 1) * slot
    base = 0x10000
    q = ctypes.c_void_p()
    assert B._lib.mrem_queue_create(depth, half, lens, ctypes.c_void_p(base), ctypes.byref(q)) == B.MREM_OK
    assert B._lib.mrem_queue_create(0, half, lens, ctypes.c_void_p(base), ctypes.byref(ctypes.c_void_p())) == B.MREM_ESHAPE
    q = q.value
    assert B.mrem_queue_size(q) == 0
    written = []
    for i in range(6):
        fp, qd, ln = B.mrem_queue_write_slot(q)
        assert fp == base + (i % (depth + 1)) * slot and qd == fp + 1024 and ln == fp + 2048
        written.append(fp)
        B.mrem_queue_publish(q)
        assert B.mrem_queue_size(q) == min(i + 1, depth)
        for age in range(B.mrem_queue_size(q)):
            assert B.mrem_queue_entry(q, age)[0] == written[i - age]          # newest first
        with pytest.raises(B.MremError):
            B.mrem_queue_entry(q, B.mrem_queue_size(q))
        # the slot being written next is never one of the readable ones
        nxt = B.mrem_queue_write_slot(q)[0]
        assert all(B.mrem_queue_entry(q, age)[0] != nxt for age in range(B.mrem_queue_size(q)))
    B.mrem_queue_destroy(q)


def test_binding_refuses_to_import_without_the_library(B, tmp_path):
    """There is no fallback path: a copy of the binding in a folder without libmrem.so must fail at
    import, naming the missing file."""
    import importlib
    import sys
    pkg = tmp_path / "mrem_without_library"
    pkg.mkdir()
    (pkg / "__init__.py").write_text("")
    (pkg / "binding.py").write_text(open(B.__file__).read())
    sys.path.insert(0, str(tmp_path))
    try:
        with pytest.raises(ImportError, match="libmrem.so is missing"):
            importlib.import_module("mrem_without_library.binding")
    finally:
        sys.path.remove(str(tmp_path))
        sys.modules.pop("mrem_without_library", None)
        sys.modules.pop("mrem_without_library.binding", None)
