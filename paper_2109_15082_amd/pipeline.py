"""Module schedules around the MREM step: sequential training of the modules (Section 4.1) and
parallel training with input queues (Section 4.2, Algorithm 1) on one GPU.

Host-side orchestration only: every tensor operation is a call into the C library
(`mrem_module_step` with its `lambda`, `mrem_module_forward`, the `mrem_queue_*` ring and the
`mrem_schedule_*` formulas).  In the parallel schedule each module has its own HIP stream (default
priority), context, parameters and workspace, so the kernels of different modules overlap on the
device the way they would on separate devices; a step ends with an event barrier between the
streams, which is the one message per step that neighbouring devices would exchange.

Queue layout: for the outputs of module n a ring of t0 + 1 slots of [batch, seq, hidden] for the
full-precision half and the same for the quantized half, plus the sequence lengths of each slot.
t0 slots are readable (the most recent t0 steps, first in first out); the extra slot is the one
being written during a step, so a module that samples the oldest entry never reads a slot while
its predecessor overwrites it.  Which entry a module samples is an argument (`slots[t][n]`, an
age: 0 = newest), drawn by the caller.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


def linear_decay_lr(lr0: float, t: int, total: int) -> float:
    """Section 5.1.2: linearly decayed rate, t = 0 .. total-1 (the library's mrem_schedule_lr)."""
    return B.mrem_schedule_lr(lr0, t, total)


def teacher_forcing_lambda(t: int, tf_steps: int) -> float:
    """Section 4.2.1: lambda_t = max(1 - t/T0, 0); 0 when teacher forcing is off (the library's mrem_schedule_lambda)."""
    return B.mrem_schedule_lambda(t, tf_steps)


class _Queue:
    """Device memory for one mrem_queue and tensor views of the addresses it hands out; the ring
    bookkeeping (write slot, publishing, entry of a given age) is the library's."""

    def __init__(self, depth: int, batch: int, seq: int, hidden: int, dtype, with_lengths: bool):
        self.shape, self.dtype, self.batch = (batch, seq, hidden), dtype, batch
        self.half_bytes = batch * seq * hidden * torch.empty(0, dtype=dtype).element_size()
        self.len_bytes = batch * 4 if with_lengths else 0
        self.mem = torch.empty(B.mrem_queue_bytes(depth, self.half_bytes, self.len_bytes), dtype=torch.uint8, device="cuda")
        self.handle = B.mrem_queue_create(depth, self.half_bytes, self.len_bytes, self.mem)

    def _views(self, addrs):
        base = self.mem.data_ptr()
        fp, qd, ln = addrs
        out = [self.mem[a - base:a - base + self.half_bytes].view(self.dtype).reshape(self.shape) for a in (fp, qd)]
        out.append(self.mem[ln - base:ln - base + self.len_bytes].view(torch.int32) if ln else None)
        return out

    def push(self, fp, qd, lengths):
        B.mrem_queue_push(self.handle, fp, qd, lengths if self.len_bytes else None)

    def written(self):
        return self._views(B.mrem_queue_write_slot(self.handle))

    def publish(self):
        B.mrem_queue_publish(self.handle)

    def entry(self, age: int):
        return self._views(B.mrem_queue_entry(self.handle, age))

    def close(self):
        if self.handle:
            B.mrem_queue_destroy(self.handle)
            self.handle = None


class ModulePipeline:
    """N consecutive modules (binding.MremModule, already loaded, initialised and calibrated)."""

    def __init__(self, modules: Sequence[B.MremModule], batch: int, seq: int, with_lengths: bool = False):
        self.modules = list(modules)
        self.batch, self.seq = batch, seq
        self.with_lengths = with_lengths
        m0 = self.modules[0]
        self.hidden, self.dtype = m0.hidden, m0.tdtype
        self.outs = [m.new_outputs(batch, seq) for m in self.modules]
        self.streams = [torch.cuda.Stream() for _ in self.modules]

    # -- one module, one step, on the current stream ---------------------------------------
    def _step(self, n: int, x_fp, x_q, lengths, lr: float, lam: float, queue: Optional[_Queue], loss_row):
        mod = self.modules[n]
        out_fp, out_q = self.outs[n]
        # Eq. 4 is part of the step: the library mixes the two inputs in the kernel that quantizes the first layer's input
        mod.step(x_fp, x_q, lr, lengths, out_fp, out_q, lam=lam if n > 0 else 0.0)
        loss_row[n].copy_(mod.loss[0], non_blocking=True)
        if queue is not None:
            queue.push(out_fp[-1], out_q[-1], lengths)

    def run_parallel(self, data: Sequence[torch.Tensor], lengths: Sequence[Optional[torch.Tensor]], slots, t0: int, total_steps: int,
                     lr0: float, tf_steps: int, concurrent: bool = True) -> torch.Tensor:
        """Algorithm 1.  data[t]: [batch, seq, hidden] device tensor entering the first module at step t;
        slots[t][n]: age of the entry module n reads at step t >= t0.  Returns losses [total_steps, N] (host)."""
        N = len(self.modules)
        queues = [_Queue(t0, self.batch, self.seq, self.hidden, self.dtype, self.with_lengths) for _ in range(N)]
        losses = torch.zeros((total_steps, N), dtype=torch.float32, device="cuda")
        main = torch.cuda.current_stream()
        for t in range(total_steps):
            lr = linear_decay_lr(lr0, t, total_steps)
            lam = teacher_forcing_lambda(t, tf_steps)
            if t < t0:
                # fill phase: one after another on the caller's stream
                x_fp = x_q = data[t]
                sl = lengths[t]
                for n in range(N):
                    self._step(n, x_fp, x_q, sl, lr, lam, queues[n], losses[t])
                    x_fp, x_q, _ = queues[n].written()
                    queues[n].publish()
                continue
            # every module reads the queues as they were after step t-1
            start = torch.cuda.Event()
            start.record(main)
            done = []
            for n in range(N):
                if n == 0:
                    x_fp = x_q = data[t]
                    sl = lengths[t]
                else:
                    x_fp, x_q, sl = queues[n - 1].entry(int(slots[t][n]))
                stream = self.streams[n] if concurrent else main
                with torch.cuda.stream(stream):
                    stream.wait_event(start)
                    self._step(n, x_fp, x_q, sl, lr, lam, queues[n], losses[t])
                    ev = torch.cuda.Event()
                    ev.record(stream)
                    done.append(ev)
            for ev in done:            # the barrier that ends the step
                main.wait_event(ev)
            for qn in queues:          # publish: first in, first out
                qn.publish()
        torch.cuda.synchronize()
        for qn in queues:
            qn.close()
        return losses.cpu()

    def run_sequential(self, data: Sequence[torch.Tensor], lengths: Sequence[Optional[torch.Tensor]], steps_per_module: int, lr0: float,
                       order=None):
        """Section 4.1: module n is trained on the outputs of the finished modules 1..n-1; order[n][t] is the
        batch module n sees at its step t (the caller's draw; default: in order, cyclically).  Returns
        (losses [N, steps_per_module] on the host, final full-precision chain outputs, final quantized chain outputs)."""
        N = len(self.modules)
        losses = torch.zeros((N, steps_per_module), dtype=torch.float32, device="cuda")
        fp_in = list(data)
        q_in = list(data)
        for n, mod in enumerate(self.modules):
            for t in range(steps_per_module):
                k = t % len(data) if order is None else int(order[n][t])
                self._step(n, fp_in[k], q_in[k], lengths[k], linear_decay_lr(lr0, t, steps_per_module), 0.0, None, losses[:, t])
            nxt_fp, nxt_q = [], []
            for k in range(len(data)):
                o_fp, o_q = mod.forward(fp_in[k], q_in[k], lengths[k])
                nxt_fp.append(o_fp[-1].clone())
                nxt_q.append(o_q[-1].clone())
            fp_in, q_in = nxt_fp, nxt_q
        torch.cuda.synchronize()
        return losses.cpu(), fp_in, q_in
