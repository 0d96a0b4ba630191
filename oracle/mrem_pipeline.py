"""Plain CPU oracle for the module schedule around the MREM step (numpy, fp64).

TEST INFRASTRUCTURE ONLY, like mrem_oracle.py, on which it builds: the product
path never imports it.

What it follows:

* Section 4.1 (end)      -- sequential training: the modules are optimised one after
                            another; module n+1 is trained on the outputs of the
                            finished modules 1..n.
* Section 4.2, Algorithm 1 -- parallel training with input queues: between module n
                            and n+1 a queue holds the outputs (full-precision and
                            quantized) of module n's most recent t0 steps, first in
                            first out; module n+1 samples an entry with replacement
                            and never waits for module n; in the first t0 steps the
                            modules run one after another to fill the queues.
* Section 4.2.1, Eq. 4   -- the quantized module's input is the convex mix
                            lambda_t f + (1 - lambda_t) f^ of a queue entry's two
                            halves, lambda_t = max(1 - t/T0, 0).

Readings taken where the paper is silent:

* a queue entry is one step's pair (f, f^) for one batch (with that batch's sequence
  lengths); both halves of a sampled entry come from the same slot, so that Eq. 4
  mixes two views of the same sequences;
* "in parallel": at step t every module sees the queues as they were after step
  t - 1 (what separate devices exchanging one message per step would see);
* the entry a module produces at step t is the pair of module outputs of that step's
  forward passes (Algorithm 2 returns them), i.e. from before the step's update;
* which entry is sampled is an input (`slots[t][n]`, an age: 0 = newest entry), so that
  both sides of a parity test draw the same numbers;
* the first module always reads the data stream (both halves equal, no mixing).

parity unpinned: none -- the pins are in tests/test_oracle_pins.py (a single module
reduces to repeated steps; the fill phase equals hand-chained steps; a queue of depth one
makes every module read its predecessor's previous output; the two inputs of module n
are what the predecessor chain produces).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import mrem_oracle as O


@dataclass
class ModuleState:
    teacher: List[Dict[str, np.ndarray]]
    student: List[Dict[str, np.ndarray]]
    adam_m: List[Dict[str, np.ndarray]]
    adam_v: List[Dict[str, np.ndarray]]
    cfg: O.Config
    updates: int = 0          # number of updates taken so far


@dataclass
class Entry:
    f_fp: np.ndarray
    f_q: np.ndarray
    seqlens: Optional[np.ndarray]


@dataclass
class Trace:
    loss: List[List[float]] = field(default_factory=list)      # loss[t][n] (run_parallel) or loss[n][t] (run_sequential)
    read_age: List[List[int]] = field(default_factory=list)    # which entry module n read at step t (-1: data)
    final_fp: Optional[List[np.ndarray]] = None                 # run_sequential: outputs of the last module's chains
    final_q: Optional[List[np.ndarray]] = None


def _one_step(ms: ModuleState, x_fp, x_q, lam: float, lr: float, batch: int, seq: int, seqlens):
    """Algorithm 2 for one module: Eq. 4 mix, both forward passes, loss, backward, update."""
    x_in = O.mix_inputs(x_fp, x_q, lam)
    ms.updates += 1
    res = O.module_step(x_fp, x_in, ms.teacher, ms.student, ms.adam_m, ms.adam_v, ms.updates, lr, ms.cfg, batch, seq, seqlens)
    return res.loss, Entry(res.f_fp[-1], res.f_q[-1], seqlens)


def run_parallel(modules: Sequence[ModuleState], data: Sequence[np.ndarray], seqlens: Sequence[Optional[np.ndarray]],
                 slots: Sequence[Sequence[int]], t0: int, total_steps: int, lr0: float, tf_steps: int,
                 batch: int, seq: int) -> Trace:
    """Algorithm 1.  data[t]: the batch [batch*seq, hidden] that enters the first module at
    step t; slots[t][n]: age of the queue entry module n (n >= 1) reads at step t >= t0,
    0 = newest, t0 - 1 = oldest.  Returns the per-step, per-module losses."""
    N = len(modules)
    queues: List[List[Entry]] = [[] for _ in range(N)]   # queues[n]: outputs of module n, newest last
    trace = Trace()
    for t in range(total_steps):
        lr = O.linear_decay_lr(lr0, t, total_steps)
        lam = O.teacher_forcing_lambda(t, tf_steps) if tf_steps > 0 else 0.0
        losses, ages, produced = [], [], []
        if t < t0:
            # fill phase: one after another, module n reads what module n-1 has just produced
            x_fp, x_q, sl = data[t], data[t], seqlens[t]
            for n in range(N):
                loss, entry = _one_step(modules[n], x_fp, x_q, lam if n > 0 else 0.0, lr, batch, seq, sl)
                queues[n].append(entry)
                losses.append(loss)
                ages.append(-1 if n == 0 else 0)
                x_fp, x_q = entry.f_fp, entry.f_q
        else:
            # every module reads the queues as they were after step t-1
            for n in range(N):
                if n == 0:
                    x_fp, x_q, sl, age = data[t], data[t], seqlens[t], -1
                else:
                    age = int(slots[t][n])
                    assert 0 <= age < len(queues[n - 1])
                    e = queues[n - 1][len(queues[n - 1]) - 1 - age]
                    x_fp, x_q, sl = e.f_fp, e.f_q, e.seqlens
                loss, entry = _one_step(modules[n], x_fp, x_q, lam if n > 0 else 0.0, lr, batch, seq, sl)
                produced.append(entry)
                losses.append(loss)
                ages.append(age)
            for n in range(N):      # first in, first out
                queues[n].append(produced[n])
                if len(queues[n]) > t0:
                    queues[n].pop(0)
        trace.loss.append(losses)
        trace.read_age.append(ages)
    return trace


def run_sequential(modules: Sequence[ModuleState], data: Sequence[np.ndarray], seqlens: Sequence[Optional[np.ndarray]],
                   steps_per_module: int, lr0: float, batch: int, seq: int, order=None) -> Trace:
    """Section 4.1: module n is trained for steps_per_module steps on the outputs of the
    finished modules 1..n-1 (full-precision chain for the teacher input, quantized chain
    for the student input).  order[n][t]: which batch module n sees at its step t (the caller's
    draw, e.g. sampled with replacement); default: in order, cyclically."""
    trace = Trace()
    fp_in = [d for d in data]
    q_in = [d for d in data]
    for n, ms in enumerate(modules):
        losses = []
        for t in range(steps_per_module):
            k = t % len(data) if order is None else int(order[n][t])
            lr = O.linear_decay_lr(lr0, t, steps_per_module)
            loss, _ = _one_step(ms, fp_in[k], q_in[k], 0.0, lr, batch, seq, seqlens[k])
            losses.append(loss)
        trace.loss.append(losses)
        # inputs of the next module: this module's two forward passes with its final parameters
        nxt_fp, nxt_q = [], []
        for k in range(len(data)):
            f_fp, _ = O.module_forward(fp_in[k], ms.teacher, ms.cfg, batch, seq, seqlens[k], quant=False)
            f_q, _ = O.module_forward(q_in[k], ms.student, ms.cfg, batch, seq, seqlens[k], quant=True)
            nxt_fp.append(f_fp[-1])
            nxt_q.append(f_q[-1])
        fp_in, q_in = nxt_fp, nxt_q
    trace.final_fp = fp_in
    trace.final_q = q_in
    return trace
