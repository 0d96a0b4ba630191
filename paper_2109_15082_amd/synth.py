"""Seeded synthetic inputs: BERT-shaped module parameters and hidden states.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no quantizer, no transformer operator, no loss).  Both the
tests of the CPU oracle and the GPU path take their inputs from here so that the
two sides see bit-identical fp32 (or bf16-representable) values.

Recipe (stands in for the calibration batches of Section 5.1: sentence pairs at
128 tokens and reading-comprehension inputs at 384 tokens, which are not
available here):

* linear weights  ~ N(0, 0.02^2), biases 0, LayerNorm gain 1 / shift 0
  (optionally jittered so that tests see non-trivial values);
* hidden states   ~ N(0, 1) per element, then each token vector is standardised
  to zero mean and unit variance (what a preceding LayerNorm would hand over);
* optional activation outliers: a seeded choice of ceil(frac * hidden) channels
  multiplied by a constant after the standardisation;
* optional key padding: sequence lengths uniform in [lo, hi].
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    seq: int
    batch: int
    act_dtype: str = "bf16"          # 'bf16' | 'f32'
    w_bits: int = 4
    a_bits: int = 8
    outlier_frac: float = 0.0
    outlier_scale: float = 20.0
    seqlen_lo: int = 0               # 0 = no padding mask
    seqlen_hi: int = 0

    @property
    def tokens(self) -> int:
        return self.seq * self.batch


#: the workloads named by the benchmark definition (index = its position there)
WORKLOADS = {
    "tiny": Workload("tiny", 1, 64, 2, 256, 32, 4, act_dtype="f32"),
    "bert_base_3l": Workload("bert_base_3l", 3, 768, 12, 3072, 128, 32),
    "bert_large_6l": Workload("bert_large_6l", 6, 1024, 16, 4096, 128, 32, outlier_frac=0.01),
    "bert_large_6l_s384": Workload("bert_large_6l_s384", 6, 1024, 16, 4096, 384, 16, outlier_frac=0.01,
                                   seqlen_lo=128, seqlen_hi=384),
    "bert_large_6l_s384_w8": Workload("bert_large_6l_s384_w8", 6, 1024, 16, 4096, 384, 16, w_bits=8,
                                      outlier_frac=0.01, seqlen_lo=128, seqlen_hi=384),
}


def make_layer_params(hidden: int, ffn: int, rng: np.random.Generator, jitter: float = 0.0) -> Dict[str, np.ndarray]:
    """fp32 parameters of one encoder layer; weights are [out, in] row-major."""
    def w(n, k):
        return (rng.standard_normal((n, k)) * 0.02).astype(np.float32)

    def vec(n, base):
        v = np.full(n, base, dtype=np.float64)
        if jitter:
            v = v + jitter * rng.standard_normal(n)
        return v.astype(np.float32)

    return {
        "w_qkv": w(3 * hidden, hidden), "b_qkv": vec(3 * hidden, 0.0),
        "w_o": w(hidden, hidden), "b_o": vec(hidden, 0.0),
        "ln1_g": vec(hidden, 1.0), "ln1_b": vec(hidden, 0.0),
        "w_1": w(ffn, hidden), "b_1": vec(ffn, 0.0),
        "w_2": w(hidden, ffn), "b_2": vec(hidden, 0.0),
        "ln2_g": vec(hidden, 1.0), "ln2_b": vec(hidden, 0.0),
    }


def make_module_params(n_layers: int, hidden: int, ffn: int, seed: int = 1234, jitter: float = 0.0) -> List[Dict[str, np.ndarray]]:
    rng = np.random.default_rng(seed)
    return [make_layer_params(hidden, ffn, rng, jitter) for _ in range(n_layers)]


def round_to_dtype(x: np.ndarray, act_dtype: str) -> np.ndarray:
    """Rounds fp32 values once to the activation storage type and returns them
    as fp32 again (a dtype conversion through the tensor library)."""
    if act_dtype == "f32":
        return np.asarray(x, dtype=np.float32)
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def make_hidden_states(batch: int, seq: int, hidden: int, seed: int = 5678, act_dtype: str = "f32",
                       outlier_frac: float = 0.0, outlier_scale: float = 20.0, outlier_seed: int = 42) -> np.ndarray:
    """[batch, seq, hidden] fp32 values already representable in act_dtype."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, seq, hidden))
    x = (x - x.mean(axis=-1, keepdims=True)) / x.std(axis=-1, keepdims=True)
    if outlier_frac > 0.0:
        n_out = int(math.ceil(outlier_frac * hidden))
        ch = np.random.default_rng(outlier_seed).choice(hidden, size=n_out, replace=False)
        x[..., ch] *= outlier_scale
    return round_to_dtype(x.astype(np.float32), act_dtype)


def make_seqlens(batch: int, lo: int, hi: int, seed: int = 99) -> Optional[np.ndarray]:
    if lo <= 0:
        return None
    return np.random.default_rng(seed).integers(lo, hi + 1, size=batch).astype(np.int32)


def make_workload_inputs(wl: Workload, weight_seed: int = 1234, input_seed: int = 5678, jitter: float = 0.0):
    """(layers, x, seqlens) for a named workload."""
    layers = make_module_params(wl.n_layers, wl.hidden, wl.ffn, weight_seed, jitter)
    x = make_hidden_states(wl.batch, wl.seq, wl.hidden, input_seed, wl.act_dtype, wl.outlier_frac, wl.outlier_scale)
    seqlens = make_seqlens(wl.batch, wl.seqlen_lo, wl.seqlen_hi)
    return layers, x, seqlens
