#!/usr/bin/env python3
"""Several consecutive modules of a BERT-shaped encoder on one GPU, synthetic data:

    python -m paper_2109_15082_amd.run_chain [--modules 4] [--layers 6] [--steps 250]
                                             [--schedule sequential|parallel] [--t0 4]

sequential (Section 4.1): every module is trained for --steps steps on the outputs of the
already trained modules before it.  parallel (Section 4.2, Algorithm 1): all modules train at
the same time for --steps steps from input queues of depth --t0 with annealed teacher forcing
over the first 40% of the steps (Section 4.2.1), each module on its own stream.  Prints one JSON
line: the end-to-end mean squared error between the full-precision and the quantized encoder
outputs before and after training, per-module first and last losses, and the training rate.
"""
import argparse
import json
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--modules", type=int, default=4)
    ap.add_argument("--layers", type=int, default=6)
    ap.add_argument("--hidden", type=int, default=1024)
    ap.add_argument("--heads", type=int, default=16)
    ap.add_argument("--ffn", type=int, default=4096)
    ap.add_argument("--seq", type=int, default=128)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--sequences", type=int, default=1024)
    ap.add_argument("--steps", type=int, default=250)
    ap.add_argument("--lr", type=float, default=1e-4)
    ap.add_argument("--schedule", choices=["sequential", "parallel"], default="sequential")
    ap.add_argument("--t0", type=int, default=4)
    ap.add_argument("--w-bits", type=int, default=4)
    ap.add_argument("--a-bits", type=int, default=8)
    ap.add_argument("--outlier-frac", type=float, default=0.01)
    args = ap.parse_args()

    import torch
    from . import binding as B, synth
    from .pipeline import ModulePipeline

    if not torch.cuda.is_available():
        raise SystemExit("run_chain: no GPU visible")
    torch.cuda.set_device(0)
    N, H = args.modules, args.hidden
    n_batches = args.sequences // args.batch
    # the calibration set: module-1 inputs, in batches
    data = []
    for k in range(n_batches):
        x = synth.make_hidden_states(args.batch, args.seq, H, 5678 + k, "bf16", args.outlier_frac, 20.0)
        data.append(torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous())
    lengths = [None] * n_batches
    # modules: seeded weights, initial weight steps, clip ranges from the full-precision chain on batch 0
    mods = []
    x_cal = data[0]
    for n in range(N):
        layers = synth.make_module_params(args.layers, H, args.ffn, 1234 + n, 0.0)
        mod = B.MremModule(args.layers, H, args.heads, args.ffn, args.batch, args.seq, act_dtype="bf16", w_bits=args.w_bits, a_bits=args.a_bits)
        mod.load(layers, layers)
        mod.init_steps()
        mod.calibrate(x_cal, None)
        o_fp, _ = mod.forward(x_cal, x_cal, None)
        x_cal = o_fp[-1].clone()
        mods.append(mod)

    def end_to_end_mse():
        tot = 0.0
        for k in range(min(4, n_batches)):
            x_fp = x_q = data[k]
            for mod in mods:
                o_fp, o_q = mod.forward(x_fp, x_q, None)
                x_fp, x_q = o_fp[-1].clone(), o_q[-1].clone()
            tot += float(((x_fp.double() - x_q.double()) ** 2).mean().item())
        return tot / min(4, n_batches)

    mse_before = end_to_end_mse()
    pipe = ModulePipeline(mods, args.batch, args.seq)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if args.schedule == "sequential":
        # every module's batches are sampled with replacement from the calibration set (seeded per module)
        order = [np.random.default_rng(4321 + n).integers(0, n_batches, size=args.steps).tolist() for n in range(N)]
        losses, _, _ = pipe.run_sequential(data, lengths, args.steps, args.lr, order)
        first, last = losses[:, 0].tolist(), losses[:, -1].tolist()
    else:
        rng = np.random.default_rng(99)
        order = rng.integers(0, n_batches, size=args.steps)          # batches sampled with replacement
        slots = rng.integers(0, args.t0, size=(args.steps, N)).tolist()
        stream = [data[i] for i in order]
        losses = pipe.run_parallel(stream, [None] * args.steps, slots, args.t0, args.steps, args.lr, int(0.4 * args.steps))
        first, last = losses[0].tolist(), losses[-1].tolist()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    mse_after = end_to_end_mse()
    module_steps = N * args.steps
    print(json.dumps({
        "schedule": args.schedule, "modules": N, "layers_per_module": args.layers, "hidden": H, "ffn": args.ffn, "seq": args.seq,
        "batch": args.batch, "sequences": args.sequences, "steps_per_module": args.steps, "w_bits": args.w_bits, "a_bits": args.a_bits,
        "end_to_end_mse_before": mse_before, "end_to_end_mse_after": mse_after,
        "loss_first_step": first, "loss_last_step": last,
        "train_seconds": dt, "module_steps_per_s": module_steps / dt, "tokens_per_s": module_steps * args.batch * args.seq / dt,
        "note": "train_seconds includes, for the sequential schedule, the forward passes that produce the next module's inputs",
        "data": "synthetic"}))
    for m in mods:
        m.close()


if __name__ == "__main__":
    main()
