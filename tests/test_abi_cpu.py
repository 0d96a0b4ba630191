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
    args = lambda ws, nbytes, batch=4, seq=32, params=fake: B._lib.mrem_module_step(
        ctx, params, fake, fake, 1, 1e-3, fake, fake, fake, fake, None, batch, seq, fake, fake, fake, None, ws, nbytes, None)
    need = B.mrem_workspace_bytes(ctx, 4, 32)
    assert args(fake, need - 1) == B.MREM_EWORKSPACE and "workspace" in B.mrem_last_error(ctx)
    assert args(None, need) == B.MREM_EINVAL
    assert args(fake, need, batch=5) == B.MREM_ESHAPE
    assert args(fake, need, seq=33) == B.MREM_ESHAPE
    assert args(fake, need, params=None) == B.MREM_EINVAL
    assert args(fake, need, params=ctypes.c_void_p(0x1004)) == B.MREM_EINVAL
    assert B._lib.mrem_quantize(None, 4, 8, 4, 1, fake, fake, None) == B.MREM_EINVAL
    assert B._lib.mrem_quantize(fake, 4, 8, 1, 1, fake, fake, None) == B.MREM_EINVAL
    B.mrem_destroy(ctx)


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
