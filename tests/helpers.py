"""Shared plumbing of the parity tests: builds the same seeded case for the CPU
oracle (numpy, fp64) and for the HIP library (torch device tensors)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

from oracle import mrem_oracle as O
from paper_2109_15082_amd import synth

MATRICES = ("w_qkv", "w_o", "w_1", "w_2")


@dataclass
class Case:
    wl: synth.Workload
    cfg: O.Config
    teacher: List[Dict[str, np.ndarray]]      # fp64 views of what the GPU teacher holds
    student: List[Dict[str, np.ndarray]]      # fp64, with steps and clip ranges
    x: np.ndarray                             # [B,S,H] fp32 values representable in act dtype
    seqlens: Optional[np.ndarray]
    layers_f32: List[Dict[str, np.ndarray]]   # the generator's fp32 parameters (teacher vector contents)
    x_q: Optional[np.ndarray] = None          # input of the quantized module when it differs from x (a layer inside a module)


def rel_err(a, ref) -> float:
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-300))


def elem_err(a, ref) -> float:
    """Largest element-wise error on the scale tol * (|ref| + max|ref|): the criterion that a single bad
    element (a wrong tile tail, one bad row) cannot hide from the way it hides in a norm."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    top = float(np.abs(ref).max()) if ref.size else 0.0
    if top == 0.0:
        return 0.0 if not np.any(a) else np.inf
    return float((np.abs(a - ref) / (np.abs(ref) + top)).max())


def conditioning(case: "Case", what: str = "forward", xq=None):
    """How far accumulation-level noise is amplified on this case, measured by the oracle alone: the same
    pass with the products formed in fp32 instead of fp64 (Config.accumulate), compared with the reference
    pass.  A code that flips at a rounding tie moves an element by a whole quantization step, and such flips
    multiply through chained quantized layers; another fp32 accumulation order (the GPU's) is expected to
    land as far from the reference as this one does.  Returns per-layer relative distances of the quantized
    module's outputs ('forward'), or (those, per-layer dicts of the norm-wise and of the element-wise relative
    distances of every gradient) ('grads')."""
    import dataclasses
    wl = case.wl
    xo = case.x.reshape(-1, wl.hidden).astype(np.float64)
    xq = xo if xq is None else np.asarray(xq, dtype=np.float64).reshape(-1, wl.hidden)   # the quantized module's input
    cfg32 = dataclasses.replace(case.cfg, accumulate="f32")
    if what == "forward":
        ref, _ = O.module_forward(xq, case.student, case.cfg, wl.batch, wl.seq, case.seqlens, quant=True)
        alt, _ = O.module_forward(xq, case.student, cfg32, wl.batch, wl.seq, case.seqlens, quant=True)
        return [rel_err(a, r) for a, r in zip(alt, ref)]
    ref = O.module_grads(xo, xq, case.teacher, case.student, case.cfg, wl.batch, wl.seq, case.seqlens)
    alt = O.module_grads(xo, xq, case.teacher, case.student, cfg32, wl.batch, wl.seq, case.seqlens)
    fwd = [rel_err(a, r) for a, r in zip(alt.f_q, ref.f_q)]
    fields = [k for k in O.TRAINABLE_FIELDS if k != "s_a"]
    grads = [{k: (rel_err(ga[k], gr[k]) if np.linalg.norm(gr[k]) > 0 else 0.0) for k in fields} for ga, gr in zip(alt.grads, ref.grads)]
    grads_elem = [{k: (elem_err(ga[k], gr[k]) if np.linalg.norm(gr[k]) > 0 else 0.0) for k in fields} for ga, gr in zip(alt.grads, ref.grads)]
    return fwd, grads, grads_elem


def mask_flip_allowance(cache, cfg: O.Config):
    """Element-wise allowances for the gradients that a straight-through mask gates directly (Section 3.1.1).
    An element that the oracle flags as lying within the storage uncertainty of a clip bound may be decided
    'inside' by one side and 'outside' by the other; its term d * 1[inside] then appears in or vanishes from
      the output gradient of the linear layer behind the quantizer -- GELU output -> first feed-forward
      projection (du = dg * gelu'(u)), Q / K / V -> query/key/value projection --
    and with it from one row of that layer's weight gradient (term d[t,n] * x^[t,:]), one entry of its bias
    gradient and one entry of its per-channel step gradient.  Returned: {field: array of the summed
    magnitudes of those terms over all flagged elements}, the exact reach of the flagged set on these fields.
    Other fields get no allowance."""
    H, nh = cfg.hidden, cfg.n_heads
    aq, wq = cache["aq"], cache["wq"]
    out = {}
    if not aq[O.AQ_G].enabled:
        return out

    def rows(delta, x_hat, wname):
        """delta[T, N]: magnitudes of the terms that may flip; x_hat[T, K]: the layer's (quantized) input."""
        a_w = np.abs(delta).T @ np.abs(x_hat)                      # [N, K]
        a_b = np.abs(delta).sum(axis=0)
        w = wq[wname]
        a_s = (a_w * np.abs(w.codes - w.v * w.inside)).sum(axis=1) if w.enabled else np.zeros(a_b.shape)
        if w.enabled and not w.per_channel:
            a_s = np.full_like(a_s, a_s.sum())
        return a_w, a_b, a_s

    # GELU-output quantizer -> first feed-forward projection
    _, near = aq[O.AQ_G].flags()
    delta = np.where(near, cache["bwd"]["dgh"] * O.gelu_grad(cache["u"]), 0.0)
    out["w_1"], out["b_1"], out["sw_1"] = rows(delta, cache["x1h"], "w_1")
    # Q, K, V quantizers -> query/key/value projection (columns: query, key, value blocks)
    cols = []
    for idx, name in ((O.AQ_Q, "dQh"), (O.AQ_K, "dKh"), (O.AQ_V, "dVh")):
        _, near = aq[idx].flags()
        cols.append(O.merge_heads(np.where(near, cache["bwd"][name], 0.0)))
    out["w_qkv"], out["b_qkv"], out["sw_qkv"] = rows(np.concatenate(cols, axis=1), cache["xh"], "w_qkv")
    return out


def elem_err_with_allowance(a, ref, allowance) -> float:
    """elem_err after taking off, per element, what the flagged mask decisions can account for."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    top = float(np.abs(ref).max()) if ref.size else 0.0
    if top == 0.0:
        return 0.0 if not np.any(a) else np.inf
    d = np.maximum(np.abs(a - ref) - np.asarray(allowance, dtype=np.float64).reshape(-1), 0.0)
    return float((d / (np.abs(ref) + top)).max())


def make_case(wl: synth.Workload, weight_seed=1234, input_seed=5678, jitter=0.05, calib_seed=None, **cfg_kw) -> Case:
    """Seeded case.  The student's weight steps are the oracle's initial steps and
    its activation clip ranges come from the oracle's calibration (on the batch
    drawn from calib_seed, default: the step's own batch)."""
    layers, x, seqlens = synth.make_workload_inputs(wl, weight_seed, input_seed, jitter)
    mode = "bf16" if wl.act_dtype == "bf16" else "f32"
    cfg = O.Config(n_layers=wl.n_layers, hidden=wl.hidden, n_heads=wl.n_heads, ffn=wl.ffn, w_bits=wl.w_bits,
                   a_bits=wl.a_bits, act_round=mode, **cfg_kw)
    student = O.to_f64(layers)
    teacher = O.to_f64(layers)
    for lp in teacher:                          # the device teacher keeps its matrices in the activation type
        for n in MATRICES:
            lp[n] = synth.round_to_dtype(lp[n].astype(np.float32), wl.act_dtype).astype(np.float64)
    for lp in student:
        for n in MATRICES:
            lp["s" + n] = O.weight_step_init(lp[n], wl.w_bits, cfg.per_channel) if wl.w_bits else np.ones(lp[n].shape[0])
        lp["s_a"], lp["z_a"] = np.ones(8), np.zeros(8)
    if wl.a_bits:
        xc = x if calib_seed is None else synth.make_hidden_states(wl.batch, wl.seq, wl.hidden, calib_seed, wl.act_dtype,
                                                                    wl.outlier_frac, wl.outlier_scale)
        cal = O.calibrate(xc.reshape(-1, wl.hidden), teacher, cfg, wl.batch, wl.seq, seqlens)
        for lp, (s, z) in zip(student, cal):
            lp["s_a"], lp["z_a"] = s.copy(), z.copy()
    return Case(wl, cfg, teacher, student, x, seqlens, layers)


def device_module(case: Case, **cfg_kw):
    """MremModule loaded with the case's parameters (steps and ranges included)."""
    import torch
    from paper_2109_15082_amd import binding as B
    wl = case.wl
    c = case.cfg
    mask = c.loss_layer_mask & 0xFFFFFFFF
    mod = B.MremModule(wl.n_layers, wl.hidden, wl.n_heads, wl.ffn, wl.batch, wl.seq, act_dtype=wl.act_dtype,
                       w_bits=wl.w_bits, a_bits=wl.a_bits, loss_layer_mask=mask, loss_mean=int(c.loss_mean),
                       ln_eps=c.ln_eps, beta1=c.beta1, beta2=c.beta2, adam_eps=c.adam_eps, weight_decay=c.weight_decay,
                       step_floor=c.step_floor, per_channel=int(c.per_channel), **cfg_kw)
    # the teacher vector holds the unrounded fp32 weights; the library rounds the matrices to the
    # activation type itself when it prepares its operand cache
    mod.load(case.student, case.layers_f32)
    return mod


def device_inputs(case: Case):
    import torch
    wl = case.wl
    td = torch.bfloat16 if wl.act_dtype == "bf16" else torch.float32
    x = torch.from_numpy(case.x).to("cuda").to(td).contiguous()
    sl = None if case.seqlens is None else torch.from_numpy(case.seqlens).to("cuda")
    return x, sl


def device_student_input(case: Case, x):
    """Device tensor of the quantized module's input: x itself unless the case has its own x_q."""
    import torch
    if case.x_q is None:
        return x
    td = torch.bfloat16 if case.wl.act_dtype == "bf16" else torch.float32
    return torch.from_numpy(np.ascontiguousarray(case.x_q, dtype=np.float32)).to("cuda").to(td).contiguous()


def fresh_moments(student):
    return ([{k: np.zeros_like(v) for k, v in lp.items()} for lp in student],
            [{k: np.zeros_like(v) for k, v in lp.items()} for lp in student])


def forward_margin(case: Case) -> float:
    """Smallest relative distance of any activation-quantizer ratio of the quantized
    forward pass to a rounding tie or clip bound (oracle only)."""
    wl = case.wl
    xo = case.x.reshape(-1, wl.hidden).astype(np.float64)
    _, caches = O.module_forward(xo, case.student, case.cfg, wl.batch, wl.seq, case.seqlens, quant=True)
    return min(a.margin for c in caches for a in c["aq"])


def make_case_with_margin(wl: synth.Workload, min_margin: float, max_tries: int = 400, calib_seed: int = 777, step_lrs=None,
                          **kw) -> Case:
    """First input seed (5678, 5679, ...) whose quantized forward pass keeps every
    ratio at least min_margin (relative) away from a discontinuity of the quantizer.
    The clip ranges are calibrated on a different batch so that no element sits
    exactly on a clip bound.  step_lrs: learning rates of consecutive steps on this batch; the
    forward pass of every one of them (the oracle runs them on a copy) must keep the margin."""
    import copy
    for i in range(max_tries):
        case = make_case(wl, input_seed=5678 + i, calib_seed=calib_seed, **kw)
        if forward_margin(case) < min_margin:
            continue
        ok = True
        if step_lrs:
            trial = copy.deepcopy(case)
            xo = trial.x.reshape(-1, wl.hidden).astype(np.float64)
            m, v = fresh_moments(trial.student)
            for t, lr in enumerate(step_lrs, start=1):
                res = O.module_step(xo, xo, trial.teacher, trial.student, m, v, t, lr, trial.cfg, wl.batch, wl.seq, trial.seqlens)
                if min(a.margin for c in res.caches for a in c["aq"]) < min_margin:
                    ok = False
                    break
        if ok:
            return case
    raise RuntimeError(f"no seed with margin {min_margin} in {max_tries} tries")


# ---------------------------------------------------------------------------------
# several consecutive modules (schedules of Section 4.1 / 4.2)
# ---------------------------------------------------------------------------------

def make_chain(wl: synth.Workload, n_modules: int, n_batches: int, **cfg_kw):
    """n_modules seeded modules (module n: weight seed 1234 + n) and n_batches input batches
    (input seed 5678 + t).  Every module's clip ranges are calibrated by the oracle on the
    full-precision chain's activations of batch 0, as a calibration pass through the modules
    in order would do.  Returns (cases, batches [n_batches][B,S,H] fp32, seqlens list)."""
    cases, batches, lens = [], [], []
    for t in range(n_batches):
        _, x, sl = synth.make_workload_inputs(wl, 1234, 5678 + t, 0.05)
        batches.append(x)
        lens.append(sl)
    x_cal = batches[0].reshape(-1, wl.hidden).astype(np.float64)
    for n in range(n_modules):
        case = make_case(wl, weight_seed=1234 + n, **cfg_kw)
        cal = O.calibrate(x_cal, case.teacher, case.cfg, wl.batch, wl.seq, lens[0])
        for lp, (s, z) in zip(case.student, cal):
            lp["s_a"], lp["z_a"] = s.copy(), z.copy()
        f_fp, _ = O.module_forward(x_cal, case.teacher, case.cfg, wl.batch, wl.seq, lens[0], quant=False)
        x_cal = f_fp[-1]
        cases.append(case)
    return cases, batches, lens


def draw_slots(total_steps: int, n_modules: int, t0: int, seed: int = 4321):
    """slots[t][n]: age (0 = newest) of the queue entry module n reads at step t."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, t0, size=(total_steps, n_modules)).tolist()
