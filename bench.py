#!/usr/bin/env python3
"""Throughput of one MREM module step (Algorithm 2) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert_large_6l]

A step = teacher forward + quantized forward + Eq. 3 loss + straight-through
backward + AdamW update of weights and step sizes, on one synthetic batch that is
already resident in HBM.  Prints ONE JSON line: tokens/s of the step (value), the time per step, the
roofline of the matrix products (bf16 and int8 launches timed with HIP events in a second pass) and
the oracle's rate on the host cores (cpu_baseline).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_INT8_PEAK_TOPS = 5000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "module_step_bert_large_6l_hbm_traffic.txt")


def measured_gemm_traffic(workload):
    """HBM bytes per matrix-product launch (read + written) as the committed rocprofv3 --pmc summary states them
    (FETCH_SIZE and WRITE_SIZE runs, each scaled by what the counter reads for a 256 MiB device copy): the line
    'traffic_bytes_per_launch: <workload> <bytes>' of profiles/module_step_bert_large_6l_hbm_traffic.txt.  Counters
    cannot be read from inside this process, so the figure comes from that file or is null."""
    try:
        for line in open(TRAFFIC_FILE):
            parts = line.strip().strip("`").split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch:" and parts[1] == workload:
                return float(parts[2])
    except OSError:
        pass
    return None


def step_flops(wl):
    """Algorithmic flops of one step: the six matrix products of every layer (four
    linear layers, Q*K^T and P*V), counted for the teacher forward, the quantized
    forward and the two backward products (input and weight gradient) of each."""
    T, H, F, S, d, nh = wl.tokens, wl.hidden, wl.ffn, wl.seq, wl.hidden // wl.n_heads, wl.n_heads
    linear = 2.0 * T * (3 * H * H + H * H + 2 * H * F)
    attn = 2.0 * wl.batch * nh * (2 * S * S * d)
    return wl.n_layers * 4.0 * (linear + attn), wl.n_layers * 4.0 * linear


def cpu_baseline(wl):
    """The oracle as it stands, on the host cores: one full step of the whole module at the full batch
    (about 16 s for bert_large_6l on the box's 16 cores; the case set-up -- the oracle's calibration pass --
    is not part of the timed step)."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import helpers as Hh
    from oracle import mrem_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    case = Hh.make_case(wl)
    xo = case.x.reshape(-1, wl.hidden).astype(np.float64)
    m, v = Hh.fresh_moments(case.student)
    t0 = time.perf_counter()
    O.module_step(xo, xo, case.teacher, case.student, m, v, 1, 1e-4, case.cfg, wl.batch, wl.seq, case.seqlens)
    dt = time.perf_counter() - t0
    return {"value": wl.tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"one full step of the {wl.n_layers}-layer module at the full batch {wl.batch} x seq {wl.seq} "
                      f"({wl.tokens} tokens) in {dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="bert_large_6l")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy before the steps (the known-size kernel that scales "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one module step on ONE GPU (the paper's per-module model parallelism reduces to "
              "one module per device); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2109_15082_amd import synth, binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    layers, x_np, seqlens = synth.make_workload_inputs(wl)
    mod = B.MremModule(wl.n_layers, wl.hidden, wl.n_heads, wl.ffn, wl.batch, wl.seq, act_dtype=wl.act_dtype,
                       w_bits=wl.w_bits, a_bits=wl.a_bits)
    mod.load(layers, layers)
    td = torch.bfloat16 if wl.act_dtype == "bf16" else torch.float32
    x = torch.from_numpy(x_np).cuda().to(td).contiguous()
    sl = None if seqlens is None else torch.from_numpy(seqlens).cuda()
    mod.init_steps()
    mod.calibrate(x, sl)
    out_fp, out_q = mod.new_outputs(wl.batch, wl.seq)
    lr0, total = 1e-4, args.steps + args.warmup
    if args.copy_probe:
        probe = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        probe_dst = torch.empty_like(probe)
        torch.cuda.synchronize()
        probe_dst.copy_(probe)   # reads 256 MiB, writes 256 MiB
    torch.cuda.synchronize()

    t = 0
    for _ in range(args.warmup):
        mod.step(x, x, lr0 * (1 - t / total), sl, out_fp, out_q)
        t += 1
    # pass 1, the timed region: K steps, nothing but the steps on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        mod.step(x, x, lr0 * (1 - t / total), sl, out_fp, out_q)
        t += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # pass 2, the same K steps again with a HIP event pair on every matrix-product launch (the pair the
    # launch itself carries: kernel begin and end, on the stream the product runs on).  Kept out of
    # pass 1 because a timed launch still costs the queue a few microseconds, which with 96 products a
    # step adds up, and because in this pass the library keeps everything on the caller's stream (in
    # pass 1 the full-precision forward pass, the weight-gradient products and the per-layer updates run
    # on a side stream beside the rest), so that every product is timed alone.
    B.mrem_profile_gemm_begin(mod.ctx)
    t1 = time.perf_counter()
    for _ in range(args.steps):
        mod.step(x, x, lr0 * (1 - (t % total) / total), sl, out_fp, out_q)
        t += 1
    torch.cuda.synchronize()
    dt_events = time.perf_counter() - t1
    (gemm_ms, gemm_flops, gemm_launches), (i8_ms, i8_ops, i8_launches) = B.mrem_profile_gemm_end(mod.ctx)
    # the bandwidth-bound kernels of the same pass: algorithmic bytes over the kernel's own duration, against HBM's 8 TB/s
    hbm_kernels = {}
    for name, (ms, nbytes, launches) in sorted(B.mrem_profile_kernels(mod.ctx).items()):
        gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        hbm_kernels[name] = {"launches_per_step": launches / args.steps, "algorithmic_bytes_per_launch": nbytes / max(launches, 1),
                             "us_per_launch": ms * 1e3 / max(launches, 1), "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": gbs / HBM_PEAK_GBS}
    losses = mod.loss.cpu().numpy()
    assert np.isfinite(losses).all(), losses

    ms_per_step = dt * 1e3 / args.steps
    tokens_per_s = wl.tokens * args.steps / dt
    flops_total, flops_linear = step_flops(wl)
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    i8_achieved = i8_ops / (i8_ms * 1e-3) / 1e12 if i8_ms > 0 else 0.0
    all_ms, all_flops, all_launches = gemm_ms + i8_ms, gemm_flops + i8_ops, gemm_launches + i8_launches
    result = {
        "metric": "module fwd+bwd tokens/s at BERT-large W4A8",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.act_dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "n_layers": wl.n_layers, "hidden": wl.hidden, "n_heads": wl.n_heads, "ffn": wl.ffn,
                   "seq_len": wl.seq, "batch": wl.batch, "w_bits": wl.w_bits, "a_bits": wl.a_bits,
                   "tokens_per_step": wl.tokens, "step_tflop": flops_total / 1e12, "loss_last_step": float(losses[0])},
        "roofline": {"bound": "mfma", "kernel": "gemm_dl_k on bf16 operands (teacher forward, input and weight gradients)",
                     "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_gemm_traffic(wl.name),
                     "traffic_unit": "bytes/launch", "traffic_source": "profiles/module_step_bert_large_6l_hbm_traffic.txt (rocprofv3 --pmc)",
                     "hbm_kernels": hbm_kernels,
                     "launches_per_step": gemm_launches / args.steps,
                     "avg_launch_us": gemm_ms * 1e3 / max(gemm_launches, 1),
                     "gemm_ms_per_step": gemm_ms / args.steps,
                     # the products of the quantized forward pass run on int8 codes and are priced against the int8 peak
                     "int8_products": {"achieved": i8_achieved, "peak": MFMA_INT8_PEAK_TOPS, "unit": "TOP/s",
                                       "frac": i8_achieved / MFMA_INT8_PEAK_TOPS, "launches_per_step": i8_launches / args.steps,
                                       "ms_per_step": i8_ms / args.steps},
                     # every product of the step against the bf16 peak
                     "all_products": {"achieved": all_flops / (all_ms * 1e-3) / 1e12 if all_ms > 0 else 0.0, "peak": MFMA_BF16_PEAK_TFLOPS,
                                      "unit": "TFLOP/s", "frac": (all_flops / (all_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS) if all_ms > 0 else 0.0,
                                      "launches_per_step": all_launches / args.steps, "ms_per_step": all_ms / args.steps},
                     "measured_on": "a second pass of the same K steps, one stream, with a HIP event pair (kernel begin, kernel end) on every product launch",
                     "ms_per_step_with_events": dt_events * 1e3 / args.steps,
                     "flops_per_launch": gemm_flops / max(gemm_launches, 1)},
        "step_tflops": flops_total / 1e12 / (ms_per_step * 1e-3),
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl)
    mod.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
