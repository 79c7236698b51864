"""Throughput of the quantized token-adaptive layer stack on one MI355X.

A "step" is one qtale_stack_forward over one batch of synthetic hidden states: for every layer the
router score, selection/compaction, gather+RMSNorm, q|k|v GEMM, rotary, attention over the executed
tokens, o GEMM, RMSNorm, gate/up GEMM with SiLU*up, down GEMM with residual and scatter.  Inputs and
quantized weights are resident in HBM before the timed region.  Prints ONE JSON line.

Workload (default): LLaMA-7B-shaped stack, 32 layers, hidden 4096, 32 heads, SwiGLU 11008, int4 group
128 round-to-nearest from N(0, 0.02) weights, router 4096 -> 1, prefill batch 8 x seq 1024,
x ~ N(0,1) bf16, execution ratio 0.5.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0


def cpu_baseline(shape, seq_len, ratio, n_layers):
    """Times the CPU oracle (as it stands) on a bounded sample: layer 0, one sequence."""
    import numpy as np
    import torch
    import synth_inputs as si
    from oracle import qtale_oracle as orc

    t = si.layer_tensors(shape, 0, 0)
    deq = {}
    for name, _, _ in shape.linear_shapes():
        c, s, z = orc.quantize_rtn(t[name].numpy(), shape.bits, shape.group)
        deq[name] = orc.dequantize(c, s, z, shape.group)
    f64 = lambda a: a.to(torch.float64).numpy()
    p = orc.LayerParams(deq["q"], deq["k"], deq["v"], deq["o"], deq["gate"], deq["up"], deq["down"],
                        f64(t["g1"]), f64(t["g2"]), t["router_w"].numpy(), 0.0)
    cfg = dict(n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
               rms_eps=shape.rms_eps, rope_base=shape.rope_base)
    x = f64(si.hidden_states(shape, seq_len, 0))
    offs, pos = si.equal_sequences(1, seq_len)
    t0 = time.perf_counter()
    orc.layer_forward(x, p, cfg, offs.numpy(), pos.numpy(), "ratio", ratio)
    dt = time.perf_counter() - t0
    cores = torch.get_num_threads()
    return {"value": seq_len / (dt * n_layers), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "oracle layer_forward (fp64 NumPy) on layer 0 and 1 sequence of %d tokens at ratio %.2f: %.2f s; "
                      "stack rate extrapolated as tokens / (%d layers x layer time)" % (seq_len, ratio, dt, n_layers)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--seq", type=int, default=1024)
    ap.add_argument("--ratio", type=float, default=0.5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only: this build uses no second GPU (run with --gpus 1)")

    import torch
    import paper_2602_10431_amd as qt
    import synth_inputs as si

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if not os.path.exists(qt.LIB_PATH):
        from paper_2602_10431_amd import build
        build.build(verbose=False)
    qt.load_library()

    shape = si.C2
    L, B, S = args.layers, args.batch, args.seq
    T = B * S
    dev = "cuda"
    cfg = qt.cfg_from_shape(shape)
    layers = []
    for l in range(L):
        t = si.layer_tensors(shape, l, 0, device=dev)
        layers.append(qt.quantize_layer(t, shape.bits, shape.group, keep_canonical=False))
        del t
    torch.cuda.synchronize()
    stack = qt.Stack(cfg, layers)
    offs, pos = si.equal_sequences(B, S)
    offs, pos = offs.to(dev), pos.to(dev)
    ws = qt.alloc_workspace(cfg, T, B, dev)
    ctx = qt.Context()
    qt.qtale_set_exec_ratio(ctx, args.ratio)
    k_exec = int(float(torch.tensor(args.ratio, dtype=torch.float32)) * T + 0.5)

    def batches(n, base):
        return [si.hidden_states(shape, T, 0, extra=base + i, device=dev) for i in range(n)]

    def run(xs):
        for x in xs:
            qt.qtale_stack_forward(ctx, stack, x, offs, pos, workspace=ws)

    run(batches(args.warmup, 1000))
    xs = batches(args.steps, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(xs)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    tokens_per_s = T * args.steps / dt

    # per-kernel durations with HIP events on the launch stream (separate pass: events perturb timing)
    xs = batches(args.steps, 0)
    qt.qtale_profile_enable(ctx, True)
    torch.cuda.synchronize()
    run(xs)
    prof = qt.qtale_profile_read(ctx)
    qt.qtale_profile_enable(ctx, False)
    kern_ms = {k: (v[0] / v[1] if v[1] else 0.0) for k, v in prof.items()}
    H, I = shape.hidden, shape.inter
    gu_flops = 2.0 * k_exec * (2 * I) * H
    gu_ms = kern_ms["gate_up_gemm"]
    achieved = gu_flops / (gu_ms * 1e-3) / 1e12 if gu_ms > 0 else 0.0
    gemm_ms = sum(kern_ms[n] for n in ("qkv_gemm", "o_gemm", "gate_up_gemm", "down_gemm"))
    gemm_flops = 2.0 * k_exec * shape.params_per_layer()
    roofline = {"bound": "mfma", "kernel": "qtale::gemm_w4a16_kernel<1,4,4,2,1,2,2,false> (gate/up GEMM with SiLU*up epilogue)",
                "achieved": achieved, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_F16_PEAK_TFLOPS, "traffic": None,
                "avg_launch_ms": gu_ms, "flops_per_launch": gu_flops,
                "all_four_gemms_tflops": gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0}

    sweep = None
    if not args.no_sweep:
        sweep = {}
        for r in (1.0, 0.8, 0.6, 0.4):
            qt.qtale_set_exec_ratio(ctx, r)
            xs = batches(3, 2000)
            run(xs[:1])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(xs[1:])
            torch.cuda.synchronize()
            sweep["%.1f" % r] = T * 2 / (time.perf_counter() - t0)
        qt.qtale_set_exec_ratio(ctx, args.ratio)

    out = {
        "metric": "tokens/s of quantized token-adaptive layer stack vs exec ratio; % HBM/MFMA peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "configs[1]: LLaMA-7B-shaped stack, %d layers, hidden 4096, 32 heads, SwiGLU 11008, "
                               "int4 group 128, prefill batch %d x seq %d, bf16 residual stream, exec ratio %.2f"
                               % (L, B, S, args.ratio),
                   "tokens_per_step": T, "executed_per_layer": k_exec},
        "roofline": roofline,
        "kernel_ms_per_launch": kern_ms,
        "tokens_per_s_vs_exec_ratio": sweep,
    }
    if not args.no_cpu_baseline:
        del xs
        out["cpu_baseline"] = cpu_baseline(shape, S, args.ratio, L)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
