"""ctypes binding of libmrem.so: argument marshalling only.

Every function has the name and the argument order of its C declaration in
include/mrem.h.  Tensors are torch tensors on the GPU (torch is used for device
memory and streams only); every step of the method runs in the HIP kernels of
the library.  Importing this module fails if the library has not been built
(python -m paper_2109_15082_amd.build): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmrem.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2109_15082_amd.build`")
_lib = C.CDLL(LIB_PATH)

MREM_OK, MREM_EINVAL, MREM_ESHAPE, MREM_EWORKSPACE, MREM_ENONFINITE, MREM_EHIP = 0, -1, -2, -3, -4, -5
MREM_BF16, MREM_FP32 = 0, 1
FIELDS = ("w_qkv", "w_o", "w_1", "w_2", "b_qkv", "b_o", "ln1_g", "ln1_b", "b_1", "b_2", "ln2_g", "ln2_b",
          "sw_qkv", "sw_o", "sw_1", "sw_2", "s_a", "z_a")
FIELD_ID = {n: i for i, n in enumerate(FIELDS)}

EXPORTS = ("mrem_create", "mrem_destroy", "mrem_last_error", "mrem_param_count", "mrem_teacher_count",
           "mrem_param_offset", "mrem_param_size", "mrem_workspace_bytes", "mrem_workspace_offset", "mrem_teacher_cache_bytes",
           "mrem_quantize", "mrem_module_init_steps", "mrem_teacher_prepare", "mrem_module_calibrate",
           "mrem_module_forward", "mrem_module_forward_static", "mrem_static_scratch_bytes", "mrem_module_step", "mrem_rem_vector_count", "mrem_rem_workspace_bytes", "mrem_rem_step", "mrem_mix_inputs", "mrem_profile_gemm_begin",
           "mrem_profile_gemm_end", "mrem_profile_kernel_count", "mrem_profile_kernel_get", "mrem_set_nonfinite_flag", "mrem_check_nonfinite", "mrem_schedule_lr", "mrem_schedule_lambda",
           "mrem_queue_bytes", "mrem_queue_create", "mrem_queue_destroy", "mrem_queue_size", "mrem_queue_write_slot", "mrem_queue_push",
           "mrem_queue_publish", "mrem_queue_entry")


class mrem_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32), ("ffn", C.c_int32),
                ("max_seq", C.c_int32), ("max_batch", C.c_int32), ("w_bits", C.c_int32), ("a_bits", C.c_int32),
                ("act_dtype", C.c_int32), ("loss_layer_mask", C.c_uint32), ("loss_mean", C.c_int32),
                ("ln_eps", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("adam_eps", C.c_float),
                ("weight_decay", C.c_float), ("step_floor", C.c_float), ("per_channel", C.c_int32)]


_vp, _i32, _i64, _f32, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
_lib.mrem_create.argtypes = [C.POINTER(mrem_config), C.POINTER(_vp)]
_lib.mrem_create.restype = C.c_int
_lib.mrem_destroy.argtypes = [_vp]
_lib.mrem_destroy.restype = None
_lib.mrem_last_error.argtypes = [_vp]
_lib.mrem_last_error.restype = C.c_char_p
_lib.mrem_param_count.argtypes = [_vp]
_lib.mrem_param_count.restype = _i64
_lib.mrem_teacher_count.argtypes = [_vp]
_lib.mrem_teacher_count.restype = _i64
_lib.mrem_param_offset.argtypes = [_vp, _i32, _i32]
_lib.mrem_param_offset.restype = _i64
_lib.mrem_param_size.argtypes = [_vp, _i32]
_lib.mrem_param_size.restype = _i64
_lib.mrem_workspace_bytes.argtypes = [_vp, _i32, _i32]
_lib.mrem_workspace_bytes.restype = _sz
_lib.mrem_workspace_offset.argtypes = [_vp, _i32, _i32, _i32, _i32]
_lib.mrem_workspace_offset.restype = _i64
_lib.mrem_teacher_cache_bytes.argtypes = [_vp]
_lib.mrem_teacher_cache_bytes.restype = _sz
_lib.mrem_quantize.argtypes = [_vp, _i64, _i64, _i32, _i32, _i32, _vp, _vp, _vp]
_lib.mrem_quantize.restype = C.c_int
_lib.mrem_module_init_steps.argtypes = [_vp, _vp, _vp]
_lib.mrem_module_init_steps.restype = C.c_int
_lib.mrem_teacher_prepare.argtypes = [_vp, _vp, _vp, _vp]
_lib.mrem_teacher_prepare.restype = C.c_int
_lib.mrem_module_calibrate.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _sz, _vp]
_lib.mrem_module_calibrate.restype = C.c_int
_lib.mrem_module_forward.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _sz, _vp]
_lib.mrem_module_forward.restype = C.c_int
_lib.mrem_module_forward_static.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp]
_lib.mrem_module_forward_static.restype = C.c_int
_lib.mrem_static_scratch_bytes.argtypes = []
_lib.mrem_static_scratch_bytes.restype = _sz
_lib.mrem_module_step.argtypes = [_vp, _vp, _vp, _vp, _i64, _f32, _f32, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp,
                                  _vp, _vp, _sz, _vp]
_lib.mrem_module_step.restype = C.c_int
_lib.mrem_rem_vector_count.argtypes = [_i64, _i64]
_lib.mrem_rem_vector_count.restype = _i64
_lib.mrem_rem_workspace_bytes.argtypes = [_vp, _i64, _i64, _i64]
_lib.mrem_rem_workspace_bytes.restype = _sz
_lib.mrem_rem_step.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.mrem_rem_step.restype = C.c_int
_lib.mrem_mix_inputs.argtypes = [_vp, _vp, _vp, _f32, _vp, _i64, _vp]
_lib.mrem_mix_inputs.restype = C.c_int


_lib.mrem_profile_gemm_begin.argtypes = [_vp]
_lib.mrem_profile_gemm_begin.restype = C.c_int
_lib.mrem_profile_gemm_end.argtypes = [_vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(_i64)]
_lib.mrem_profile_gemm_end.restype = C.c_int
_lib.mrem_profile_kernel_count.argtypes = [_vp]
_lib.mrem_profile_kernel_count.restype = _i32
_lib.mrem_profile_kernel_get.argtypes = [_vp, _i32, C.c_char_p, _i32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(_i64)]
_lib.mrem_profile_kernel_get.restype = C.c_int
_lib.mrem_set_nonfinite_flag.argtypes = [_vp, _vp]
_lib.mrem_set_nonfinite_flag.restype = C.c_int
_lib.mrem_check_nonfinite.argtypes = [_vp, _vp]
_lib.mrem_check_nonfinite.restype = C.c_int
_lib.mrem_schedule_lr.argtypes = [C.c_double, _i64, _i64]
_lib.mrem_schedule_lr.restype = C.c_double
_lib.mrem_schedule_lambda.argtypes = [_i64, _i64]
_lib.mrem_schedule_lambda.restype = C.c_double
_lib.mrem_queue_bytes.argtypes = [_i32, _sz, _sz]
_lib.mrem_queue_bytes.restype = _sz
_lib.mrem_queue_create.argtypes = [_i32, _sz, _sz, _vp, C.POINTER(_vp)]
_lib.mrem_queue_create.restype = C.c_int
_lib.mrem_queue_destroy.argtypes = [_vp]
_lib.mrem_queue_destroy.restype = None
_lib.mrem_queue_size.argtypes = [_vp]
_lib.mrem_queue_size.restype = _i32
_lib.mrem_queue_write_slot.argtypes = [_vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_vp)]
_lib.mrem_queue_write_slot.restype = C.c_int
_lib.mrem_queue_push.argtypes = [_vp, _vp, _vp, _vp, _sz, _sz, _vp]
_lib.mrem_queue_push.restype = C.c_int
_lib.mrem_queue_publish.argtypes = [_vp]
_lib.mrem_queue_publish.restype = C.c_int
_lib.mrem_queue_entry.argtypes = [_vp, _i32, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_vp)]
_lib.mrem_queue_entry.restype = C.c_int


class MremError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"mrem status {status}: {message}")
        self.status = status


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor required")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor required")
    return t.data_ptr()


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return getattr(stream, "cuda_stream", stream)


def _check(status: int, ctx=None):
    if status != MREM_OK:
        raise MremError(status, mrem_last_error(ctx))


def mrem_last_error(ctx=None) -> str:
    return (_lib.mrem_last_error(ctx) or b"").decode()


def mrem_create(**kw) -> int:
    """Returns an opaque context handle.  Keyword arguments are the fields of mrem_config."""
    cfg = mrem_config(loss_layer_mask=0xFFFFFFFF, loss_mean=1, ln_eps=1e-12, beta1=0.9, beta2=0.999, adam_eps=1e-8,
                      weight_decay=0.01, step_floor=1e-8, w_bits=4, a_bits=8, act_dtype=MREM_BF16, per_channel=1)
    for k, v in kw.items():
        if not hasattr(cfg, k):
            raise TypeError(f"unknown mrem_config field {k}")
        setattr(cfg, k, v)
    out = _vp()
    _check(_lib.mrem_create(C.byref(cfg), C.byref(out)))
    return out.value


def mrem_destroy(ctx) -> None:
    _lib.mrem_destroy(ctx)


def mrem_param_count(ctx) -> int:
    return _lib.mrem_param_count(ctx)


def mrem_teacher_count(ctx) -> int:
    return _lib.mrem_teacher_count(ctx)


def mrem_param_offset(ctx, layer: int, field) -> int:
    return _lib.mrem_param_offset(ctx, layer, FIELD_ID[field] if isinstance(field, str) else field)


def mrem_param_size(ctx, field) -> int:
    return _lib.mrem_param_size(ctx, FIELD_ID[field] if isinstance(field, str) else field)


def mrem_workspace_bytes(ctx, batch: int, seq: int) -> int:
    return _lib.mrem_workspace_bytes(ctx, batch, seq)


MREM_WS_WCODES8, MREM_WS_WCODES, MREM_WS_QKV, MREM_WS_XCODES8 = 0, 4, 8, 9


def mrem_workspace_offset(ctx, batch: int, seq: int, layer: int, item: int) -> int:
    return _lib.mrem_workspace_offset(ctx, batch, seq, layer, item)


def mrem_teacher_cache_bytes(ctx) -> int:
    return _lib.mrem_teacher_cache_bytes(ctx)


def mrem_quantize(w, N, K, bits, per_channel, init_scale, scale, codes, stream=None) -> None:
    _check(_lib.mrem_quantize(_ptr(w), N, K, bits, per_channel, init_scale, _ptr(scale), _ptr(codes), _stream(stream)))


def mrem_module_init_steps(ctx, params, stream=None) -> None:
    _check(_lib.mrem_module_init_steps(ctx, _ptr(params), _stream(stream)), ctx)


def mrem_teacher_prepare(ctx, teacher, cache, stream=None) -> None:
    _check(_lib.mrem_teacher_prepare(ctx, _ptr(teacher), _ptr(cache), _stream(stream)), ctx)


def mrem_module_calibrate(ctx, params, teacher, teacher_cache, x_fp, seqlens, batch, seq, workspace, stream=None) -> None:
    _check(_lib.mrem_module_calibrate(ctx, _ptr(params), _ptr(teacher), _ptr(teacher_cache), _ptr(x_fp), _ptr(seqlens),
                                      batch, seq, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)), ctx)


def mrem_module_forward(ctx, params, teacher, teacher_cache, x_fp, x_q, seqlens, batch, seq, per_layer_fp, per_layer_q,
                        workspace, stream=None) -> None:
    _check(_lib.mrem_module_forward(ctx, _ptr(params), _ptr(teacher), _ptr(teacher_cache), _ptr(x_fp), _ptr(x_q),
                                    _ptr(seqlens), batch, seq, _ptr(per_layer_fp), _ptr(per_layer_q), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)), ctx)


def mrem_static_scratch_bytes() -> int:
    return _lib.mrem_static_scratch_bytes()


def mrem_module_forward_static(ctx, params, teacher, teacher_cache, x_fp, x_q, seqlens, batch, seq, per_layer_fp, per_layer_q,
                               stream=None) -> None:
    _check(_lib.mrem_module_forward_static(ctx, _ptr(params), _ptr(teacher), _ptr(teacher_cache), _ptr(x_fp), _ptr(x_q),
                                           _ptr(seqlens), batch, seq, _ptr(per_layer_fp), _ptr(per_layer_q), _stream(stream)), ctx)


def mrem_module_step(ctx, params, adam_m, adam_v, step_index, lr, lam, teacher, teacher_cache, x_fp, x_q, seqlens, batch, seq,
                     loss_out, per_layer_fp, per_layer_q, grads_out, workspace, stream=None) -> None:
    _check(_lib.mrem_module_step(ctx, _ptr(params), _ptr(adam_m), _ptr(adam_v), step_index, lr, lam, _ptr(teacher),
                                 _ptr(teacher_cache), _ptr(x_fp), _ptr(x_q), _ptr(seqlens), batch, seq, _ptr(loss_out),
                                 _ptr(per_layer_fp), _ptr(per_layer_q), _ptr(grads_out), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)), ctx)


def mrem_rem_vector_count(N: int, K: int) -> int:
    return _lib.mrem_rem_vector_count(N, K)


def mrem_rem_workspace_bytes(ctx, T: int, N: int, K: int) -> int:
    return _lib.mrem_rem_workspace_bytes(ctx, T, N, K)


def mrem_rem_step(ctx, T, N, K, vec, adam_m, adam_v, step_index, lr, w_fp, a_fp, a_q, loss_out, y_fp, y_q, grads_out, workspace,
                  stream=None) -> None:
    _check(_lib.mrem_rem_step(ctx, T, N, K, _ptr(vec), _ptr(adam_m), _ptr(adam_v), step_index, lr, _ptr(w_fp), _ptr(a_fp), _ptr(a_q),
                              _ptr(loss_out), _ptr(y_fp), _ptr(y_q), _ptr(grads_out), _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _stream(stream)), ctx)


def mrem_mix_inputs(ctx, x_fp, x_q, lam, out, n, stream=None) -> None:
    _check(_lib.mrem_mix_inputs(ctx, _ptr(x_fp), _ptr(x_q), lam, _ptr(out), n, _stream(stream)), ctx)


def mrem_profile_gemm_begin(ctx) -> None:
    _check(_lib.mrem_profile_gemm_begin(ctx), ctx)


def mrem_profile_gemm_end(ctx):
    """((ms, flops, launches) of the products on bf16 operands, the same for int8 operands) since _begin."""
    ms, fl, n = (C.c_double * 2)(), (C.c_double * 2)(), (_i64 * 2)()
    _check(_lib.mrem_profile_gemm_end(ctx, ms, fl, n), ctx)
    return (ms[0], fl[0], n[0]), (ms[1], fl[1], n[1])


def mrem_profile_kernels(ctx):
    """{kernel name: (ms, algorithmic bytes, launches)} of the bandwidth-bound kernels of the last timed interval."""
    out = {}
    for i in range(_lib.mrem_profile_kernel_count(ctx)):
        name = C.create_string_buffer(64)
        ms, nb, n = C.c_double(), C.c_double(), _i64()
        _check(_lib.mrem_profile_kernel_get(ctx, i, name, 64, C.byref(ms), C.byref(nb), C.byref(n)), ctx)
        out[name.value.decode()] = (ms.value, nb.value, n.value)
    return out


def mrem_set_nonfinite_flag(ctx, flag) -> None:
    _check(_lib.mrem_set_nonfinite_flag(ctx, _ptr(flag)), ctx)


def mrem_check_nonfinite(ctx, stream=None) -> None:
    _check(_lib.mrem_check_nonfinite(ctx, _stream(stream)), ctx)


def mrem_schedule_lr(lr0: float, t: int, total: int) -> float:
    return _lib.mrem_schedule_lr(lr0, t, total)


def mrem_schedule_lambda(t: int, tf_steps: int) -> float:
    return _lib.mrem_schedule_lambda(t, tf_steps)


def mrem_queue_bytes(depth: int, half_bytes: int, lengths_bytes: int) -> int:
    return _lib.mrem_queue_bytes(depth, half_bytes, lengths_bytes)


def mrem_queue_create(depth: int, half_bytes: int, lengths_bytes: int, device_mem) -> int:
    out = _vp()
    _check(_lib.mrem_queue_create(depth, half_bytes, lengths_bytes, _ptr(device_mem), C.byref(out)))
    return out.value


def mrem_queue_destroy(q) -> None:
    _lib.mrem_queue_destroy(q)


def mrem_queue_size(q) -> int:
    return _lib.mrem_queue_size(q)


def _three(fn, *args):
    a, b, c = _vp(), _vp(), _vp()
    _check(fn(*args, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def mrem_queue_write_slot(q):
    """Device addresses (fp half, quantized half, lengths or None) of the slot being written."""
    return _three(_lib.mrem_queue_write_slot, q)


def mrem_queue_push(q, fp, qd, lengths, stream=None) -> None:
    nb = fp.numel() * fp.element_size()
    lb = 0 if lengths is None else lengths.numel() * lengths.element_size()
    _check(_lib.mrem_queue_push(q, _ptr(fp), _ptr(qd), _ptr(lengths), nb, lb, _stream(stream)))


def mrem_queue_publish(q) -> None:
    _check(_lib.mrem_queue_publish(q))


def mrem_queue_entry(q, age: int):
    """Device addresses (fp half, quantized half, lengths or None) of the entry of that age (0 = newest)."""
    return _three(_lib.mrem_queue_entry, q, age)


# ------------------------------------------------------------------------------
# buffer plumbing for callers (no arithmetic of the method here)
# ------------------------------------------------------------------------------

def pack_params(ctx, layers, device="cuda") -> torch.Tensor:
    """Flat fp32 vector in the library's layout from a list of per-layer dicts of
    numpy arrays (missing fields, e.g. step sizes of a teacher, stay 0)."""
    import numpy as np
    flat = np.zeros(mrem_param_count(ctx), dtype=np.float32)
    for l, lp in enumerate(layers):
        for name, arr in lp.items():
            off = mrem_param_offset(ctx, l, name)
            n = mrem_param_size(ctx, name)
            flat[off:off + n] = np.asarray(arr, dtype=np.float32).reshape(-1)
    return torch.from_numpy(flat).to(device)


def unpack_params(ctx, flat: torch.Tensor, n_layers: int, shapes=None):
    """Inverse of pack_params: list of per-layer dicts of numpy arrays (1-D unless shapes given)."""
    host = flat.detach().float().cpu().numpy()
    out = []
    for l in range(n_layers):
        d = {}
        for name in FIELDS:
            off = mrem_param_offset(ctx, l, name)
            n = mrem_param_size(ctx, name)
            a = host[off:off + n].copy()
            if shapes and name in shapes:
                a = a.reshape(shapes[name])
            d[name] = a
        out.append(d)
    return out


class MremModule:
    """Owns the device buffers of one module and forwards to the C entry points."""

    def __init__(self, n_layers, hidden, n_heads, ffn, max_batch, max_seq, act_dtype="bf16", **cfg):
        self.n_layers, self.hidden, self.n_heads, self.ffn = n_layers, hidden, n_heads, ffn
        self.act_dtype = act_dtype
        self.tdtype = torch.bfloat16 if act_dtype == "bf16" else torch.float32
        self.ctx = mrem_create(n_layers=n_layers, hidden=hidden, n_heads=n_heads, ffn=ffn, max_batch=max_batch,
                               max_seq=max_seq, act_dtype=MREM_BF16 if act_dtype == "bf16" else MREM_FP32, **cfg)
        self.max_batch, self.max_seq = max_batch, max_seq
        n = mrem_param_count(self.ctx)
        dev = "cuda"
        self.params = torch.zeros(n, dtype=torch.float32, device=dev)
        self.teacher = torch.zeros(n, dtype=torch.float32, device=dev)
        self.adam_m = torch.zeros(n, dtype=torch.float32, device=dev)
        self.adam_v = torch.zeros(n, dtype=torch.float32, device=dev)
        self.teacher_cache = torch.empty(mrem_teacher_cache_bytes(self.ctx), dtype=torch.uint8, device=dev)
        self.workspace = torch.empty(mrem_workspace_bytes(self.ctx, max_batch, max_seq), dtype=torch.uint8, device=dev)
        self.loss = torch.zeros(1 + n_layers, dtype=torch.float32, device=dev)
        self.step_index = 0

    def shapes(self):
        H, F = self.hidden, self.ffn
        return {"w_qkv": (3 * H, H), "w_o": (H, H), "w_1": (F, H), "w_2": (H, F)}

    def load(self, student_layers, teacher_layers=None):
        self.params.copy_(pack_params(self.ctx, student_layers))
        self.teacher.copy_(pack_params(self.ctx, teacher_layers if teacher_layers is not None else student_layers))
        mrem_teacher_prepare(self.ctx, self.teacher, self.teacher_cache)

    def init_steps(self):
        mrem_module_init_steps(self.ctx, self.params)

    def calibrate(self, x_fp, seqlens=None):
        b, s = x_fp.shape[0], x_fp.shape[1]
        mrem_module_calibrate(self.ctx, self.params, self.teacher, self.teacher_cache, x_fp, seqlens, b, s, self.workspace)

    def new_outputs(self, batch, seq):
        shape = (self.n_layers, batch, seq, self.hidden)
        return (torch.empty(shape, dtype=self.tdtype, device="cuda"), torch.empty(shape, dtype=self.tdtype, device="cuda"))

    def forward(self, x_fp, x_q, seqlens=None, out_fp=None, out_q=None):
        b, s = x_fp.shape[0], x_fp.shape[1]
        if out_fp is None or out_q is None:
            out_fp, out_q = self.new_outputs(b, s)
        mrem_module_forward(self.ctx, self.params, self.teacher, self.teacher_cache, x_fp, x_q, seqlens, b, s, out_fp, out_q,
                            self.workspace)
        return out_fp, out_q

    def step(self, x_fp, x_q, lr, seqlens=None, out_fp=None, out_q=None, grads_out=None, lam=0.0):
        b, s = x_fp.shape[0], x_fp.shape[1]
        if out_fp is None or out_q is None:
            out_fp, out_q = self.new_outputs(b, s)
        self.step_index += 1
        mrem_module_step(self.ctx, self.params, self.adam_m, self.adam_v, self.step_index, lr, lam, self.teacher,
                         self.teacher_cache, x_fp, x_q, seqlens, b, s, self.loss, out_fp, out_q, grads_out, self.workspace)
        return out_fp, out_q

    def close(self):
        if self.ctx:
            mrem_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
