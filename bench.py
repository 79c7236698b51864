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


def _blas_threads():
    """Threads the NumPy BLAS pool will use (the oracle's matrix products run there)."""
    try:
        import threadpoolctl
        n = [d["num_threads"] for d in threadpoolctl.threadpool_info() if d.get("user_api") == "blas"]
        return max(n) if n else 1
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(shape, n_seq, seq_len, ratio, n_layers, reps=3):
    """Times the CPU oracle (as it stands) on a bounded sample: layer 0 on whole batches with the BLAS pool as
    NumPy finds it, then the same layer on a quarter batch with the pool limited to one thread."""
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
    T = n_seq * seq_len
    xs = [f64(si.hidden_states(shape, T, 0, extra=i)) for i in range(reps)]
    offs, pos = si.equal_sequences(n_seq, seq_len)
    cores = _blas_threads()
    t0 = time.perf_counter()
    for x in xs:
        orc.layer_forward(x, p, cfg, offs.numpy(), pos.numpy(), "ratio", ratio)
    dt = (time.perf_counter() - t0) / reps
    out = {"value": T / (dt * n_layers), "unit": "tokens/s", "cores": cores, "kind": "oracle",
           "sample": "oracle layer_forward (fp64 NumPy, BLAS pool of %d threads) on layer 0 and %d batches of %d x %d "
                     "tokens at ratio %.2f: %.2f s per batch; stack rate extrapolated as tokens / (%d layers x layer time)"
                     % (cores, reps, n_seq, seq_len, ratio, dt, n_layers)}
    # one core: the same layer on a quarter of the sequences, BLAS pool limited to a single thread
    try:
        import threadpoolctl
        n1 = max(1, n_seq // 4)
        o1, p1 = si.equal_sequences(n1, seq_len)
        x1 = xs[0][:n1 * seq_len]
        with threadpoolctl.threadpool_limits(limits=1):
            t0 = time.perf_counter()
            orc.layer_forward(x1, p, cfg, o1.numpy(), p1.numpy(), "ratio", ratio)
            dt1 = time.perf_counter() - t0
        out["one_core"] = {"value": n1 * seq_len / (dt1 * n_layers), "unit": "tokens/s", "cores": 1,
                           "sample": "same layer on %d x %d tokens with the BLAS pool limited to 1 thread: %.2f s; "
                                     "extrapolated to %d layers" % (n1, seq_len, dt1, n_layers)}
    except Exception as e:      # threadpoolctl missing: report that instead of a number
        out["one_core"] = {"value": None, "note": "threadpoolctl unavailable: %s" % e}
    return out


def recorded_traffic():
    """HBM-side bytes per launch of the gate/up GEMM from the committed rocprofv3 --pmc summary, or None
    when the kernel sources have changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "gate_up_gemm_7b_prefill_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if not line.startswith("#") and ":" in line:
            k, v = line.split(":", 1)
            vals[k.strip()] = v.strip()
    h = hashlib.sha256()
    for rel in ("gemm_w4a16.hip", "gemm_common.h", "qtale_dev.h"):
        h.update(open(os.path.join(ROOT, "paper_2602_10431_amd", "csrc", rel), "rb").read())
    if vals.get("kernel_sources_sha256") != h.hexdigest():
        return None
    return float(vals["traffic_bytes_per_launch"])


def decode_section(qt, si, torch, layers, L, B=64, ctx_len=2048, steps=256, bits=4, ratios=(1.0, 0.8, 0.6, 0.4),
                   base=None, kv_distinct=None, graph_steps=32, label="configs[2]"):
    """Decode steps of a stack: batch B, ctx_len cached entries per sequence and layer (random fp16 K/V), `steps`
    generated steps per ratio, execution ratio changed at run time (no requantization).  Every input of the timed
    loops (hidden states, positions) is staged on the GPU beforehand: the loops contain library calls only.
    kv_distinct: number of distinct per-layer K/V buffers; layers beyond it alias them round-robin (each layer keeps
    its own length counters) - for stacks whose caches exceed HBM."""
    import dataclasses
    dev = "cuda"
    base = base or si.C2
    shape = dataclasses.replace(base, bits=bits, act_dtype="fp16")
    cfg = qt.cfg_from_shape(shape)
    nkv, d = shape.n_kv_heads, shape.head_dim
    fp16_layers = []
    for lw in layers:                                  # same quantized weights, fp16 gains for an fp16 stream
        fp16_layers.append(qt.LayerWeights(lw.lin["q"], lw.lin["k"], lw.lin["v"], lw.lin["o"], lw.lin["gate"],
                                           lw.lin["up"], lw.lin["down"], lw.norm1.to(torch.float16),
                                           lw.norm2.to(torch.float16), lw.router_w, lw.router_b))
    cap = ctx_len + steps + 8
    n_buf = L if kv_distinct is None else min(L, kv_distinct)
    bufs = []
    for l in range(n_buf):
        k = torch.randn(B, nkv, cap, d, device=dev, dtype=torch.float16)       # [B][kv heads][cap][head_dim]
        v = torch.randn(B, nkv, cap, d, device=dev, dtype=torch.float16)
        bufs.append((k, v))
    kvs = [qt.KVCache(bufs[l % n_buf][0], bufs[l % n_buf][1], torch.full((B,), ctx_len, dtype=torch.int32, device=dev))
           for l in range(L)]
    stack = qt.Stack(cfg, fp16_layers, kvs)
    offs = torch.arange(0, B + 1, dtype=torch.int32, device=dev)
    ws = qt.alloc_workspace(cfg, B, B, dev)
    ctx = qt.Context()
    n_x = min(steps, 16)                                # distinct hidden-state batches, reused round-robin
    xs = [si.hidden_states(shape, B, 0, slot="x_step", extra=i, device=dev) for i in range(n_x)]
    x_run = [torch.empty_like(xs[0]) for _ in range(steps)]
    pos_run = [torch.full((B,), ctx_len + i, dtype=torch.int32, device=dev) for i in range(steps)]
    H = shape.hidden
    w_bytes = shape.params_per_layer() * bits // 8 + 4 * (shape.params_per_layer() // shape.group)
    res = {}
    for r in ratios:
        qt.qtale_set_exec_ratio(ctx, r)                 # runtime change: no requantization
        k_exec = int(float(torch.tensor(r, dtype=torch.float32)) * B + 0.5)

        def stage(n):
            for kv in kvs:
                kv.kv_len.fill_(ctx_len)
            for i in range(n):
                x_run[i].copy_(xs[i % n_x])             # the stack updates x in place: fresh copies per step
            torch.cuda.synchronize()

        def run(n, profile=False):
            stage(n)
            qt.qtale_profile_enable(ctx, profile)
            t0 = time.perf_counter()
            for i in range(n):
                qt.qtale_stack_forward(ctx, stack, x_run[i], offs, pos_run[i], workspace=ws)
            torch.cuda.synchronize()
            return time.perf_counter() - t0

        def run_graph(n):
            # the same step replayed from one HIP graph (pointers baked in): the replay loop contains graph launches
            # only, so x is whatever the previous replay left and the positions stay at ctx_len (cache lengths still
            # advance on the device); same kernels and shapes as the eager steps
            stage(1)
            graph = qt.StackGraph(ctx, stack, x_run[0], offs, pos_run[0], workspace=ws)
            best = None
            for _ in range(2):
                stage(1)
                t0 = time.perf_counter()
                for i in range(n):
                    graph.launch()
                torch.cuda.synchronize()
                best = time.perf_counter() - t0
            return best

        run(min(steps, 8))
        dt = run(steps)
        dt_graph = run_graph(min(steps, graph_steps)) if graph_steps else None
        n_prof = min(steps, 8)
        run(n_prof, True)
        prof = qt.qtale_profile_read(ctx)
        qt.qtale_profile_enable(ctx, False)
        n_layer_calls = prof["attention"][1]            # per layer call: inside a stack the router of layers 1.. is fused away
        ms = {k: (v[0] / n_layer_calls if n_layer_calls else 0.0) for k, v in prof.items()}
        lin_ms = ms["qkv_gemm"] + ms["o_gemm"] + ms["gate_up_gemm"] + ms["down_gemm"]
        kv_bytes = k_exec * (ctx_len + n_prof / 2.0) * 2 * nkv * d * 2
        res["%.1f" % r] = {"tokens_per_s": B * steps / dt, "ms_per_step": dt * 1e3 / steps,
                           "hip_graph_ms_per_step": dt_graph * 1e3 / min(steps, graph_steps) if dt_graph else None,
                           "executed_per_layer": k_exec,
                           "attention_ms": ms["attention"], "attention_GBps": kv_bytes / (ms["attention"] * 1e6),
                           "attention_frac_of_hbm_peak": kv_bytes / (ms["attention"] * 1e6) / HBM_PEAK_GBS,
                           "linears_ms": lin_ms, "weight_stream_GBps": w_bytes / (lin_ms * 1e6),
                           "linears_frac_of_hbm_peak": w_bytes / (lin_ms * 1e6) / HBM_PEAK_GBS,
                           "small_kernels_ms": sum(ms[k] for k in ("router", "select", "norm1", "rope_append", "norm2"))}
    del kvs, bufs, stack
    torch.cuda.empty_cache()
    alias = "" if n_buf == L else (", K/V storage of %d layers aliased round-robin by the %d layers (one layer's K/V, "
                                   "%.1f GB, is far beyond the 256 MB memory-side cache)" % (n_buf, L, 2.0 * B * nkv * cap * d * 2 / 1e9))
    return {"workload": "%s: %d-layer stack (hidden %d, %d/%d heads, SwiGLU %d, int%d) in decode, batch %d, %d cached K/V "
                        "entries per sequence and layer (random fp16), %d steps per ratio, fp16 stream%s; per-kernel "
                        "times from HIP events (they include launch gaps)"
                        % (label, L, H, shape.n_heads, nkv, shape.inter, bits, B, ctx_len, steps, alias),
            "hbm_peak_GBps": HBM_PEAK_GBS, "by_exec_ratio": res}


def quantized_stack(qt, si, torch, shape, L, bits=None):
    layers = []
    for l in range(L):
        t = si.layer_tensors(shape, l, 0, device="cuda")
        layers.append(qt.quantize_layer(t, bits or shape.bits, shape.group, keep_canonical=False))
        del t
    torch.cuda.synchronize()
    return layers


def prefill_section(qt, si, torch, shape, layers, B, S, ratios, label, steps=3):
    """Prefill steps of another stack (configs[3], configs[4]): tokens/s per ratio, and the gate/up GEMM and
    attention rates from HIP events at the first ratio."""
    dev = "cuda"
    L = len(layers)
    cfg = qt.cfg_from_shape(shape)
    stack = qt.Stack(cfg, layers)
    T = B * S
    offs, pos = si.equal_sequences(B, S)
    offs, pos = offs.to(dev), pos.to(dev)
    ws = qt.alloc_workspace(cfg, T, B, dev)
    ctx = qt.Context()
    out = {"workload": "%s: %d-layer stack (hidden %d, %d/%d heads, SwiGLU %d, int%d group %d), prefill %d x %d, %s stream"
                       % (label, L, shape.hidden, shape.n_heads, shape.n_kv_heads, shape.inter, shape.bits, shape.group, B, S,
                          shape.act_dtype), "by_exec_ratio": {}}
    for i, r in enumerate(ratios):
        qt.qtale_set_exec_ratio(ctx, r)
        k_exec = int(float(torch.tensor(r, dtype=torch.float32)) * T + 0.5)
        xs = [si.hidden_states(shape, T, 0, extra=8000 + j, device=dev) for j in range(steps + 1)]
        qt.qtale_stack_forward(ctx, stack, xs[0], offs, pos, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for x in xs[1:]:
            qt.qtale_stack_forward(ctx, stack, x, offs, pos, workspace=ws)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        entry = {"tokens_per_s": T / dt, "ms_per_step": dt * 1e3, "executed_per_layer": k_exec}
        if i == 0:
            x = si.hidden_states(shape, T, 0, extra=8100, device=dev)
            qt.qtale_profile_enable(ctx, True)
            qt.qtale_stack_forward(ctx, stack, x, offs, pos, workspace=ws)
            prof = qt.qtale_profile_read(ctx)
            qt.qtale_profile_enable(ctx, False)
            ms = {k: (v[0] / v[1] if v[1] else 0.0) for k, v in prof.items()}
            gu = 2.0 * k_exec * 2 * shape.inter * shape.hidden
            n_b = k_exec / B                                       # executed tokens per sequence (equal sequences, on average)
            att = 4.0 * n_b * n_b / 2 * shape.n_heads * shape.head_dim * B
            entry["kernel_ms_per_launch"] = ms
            entry["gate_up_gemm_TFLOPs"] = gu / (ms["gate_up_gemm"] * 1e-3) / 1e12
            entry["gate_up_gemm_frac_of_mfma_peak"] = entry["gate_up_gemm_TFLOPs"] / MFMA_F16_PEAK_TFLOPS
            entry["attention_TFLOPs_causal"] = att / (ms["attention"] * 1e-3) / 1e12
            entry["attention_share_of_layer"] = ms["attention"] / sum(ms.values())
        out["by_exec_ratio"]["%.1f" % r] = entry
        del xs
    del ws, stack
    torch.cuda.empty_cache()
    return out


def int3_section(qt, si, torch, shape4, L, B, S, ratio, no_decode, layers4=None):
    """The 3-bit variant of the same workload (Sec. 4.1 evaluates 4-bit and 3-bit weights): prefill step
    and gate/up GEMM rate, then two decode ratios."""
    import dataclasses
    dev = "cuda"
    shape = dataclasses.replace(shape4, bits=3)
    cfg = qt.cfg_from_shape(shape)
    layers = []
    for l in range(L):
        t = si.layer_tensors(shape, l, 0, device=dev)
        layers.append(qt.quantize_layer(t, 3, shape.group, keep_canonical=False))
        del t
    stack = qt.Stack(cfg, layers)
    T = B * S
    offs, pos = si.equal_sequences(B, S)
    offs, pos = offs.to(dev), pos.to(dev)
    ws = qt.alloc_workspace(cfg, T, B, dev)
    ctx = qt.Context()
    qt.qtale_set_exec_ratio(ctx, ratio)
    k_exec = int(float(torch.tensor(ratio, dtype=torch.float32)) * T + 0.5)
    xs = [si.hidden_states(shape, T, 0, extra=3000 + i, device=dev) for i in range(4)]
    qt.qtale_stack_forward(ctx, stack, xs[0], offs, pos, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for x in xs[1:]:
        qt.qtale_stack_forward(ctx, stack, x, offs, pos, workspace=ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / 3
    xs = [si.hidden_states(shape, T, 0, extra=3000 + i, device=dev) for i in range(2)]
    qt.qtale_profile_enable(ctx, True)
    for x in xs:
        qt.qtale_stack_forward(ctx, stack, x, offs, pos, workspace=ws)
    prof = qt.qtale_profile_read(ctx)
    qt.qtale_profile_enable(ctx, False)
    gu_ms = prof["gate_up_gemm"][0] / prof["gate_up_gemm"][1]
    out = {"workload": "same stack and batch with 3-bit group-128 codes (0.375 B/weight)",
           "prefill_tokens_per_s": T / dt, "prefill_ms_per_step": dt * 1e3,
           "gate_up_gemm_ms": gu_ms, "gate_up_gemm_TFLOPs": 2.0 * k_exec * 2 * shape.inter * shape.hidden / (gu_ms * 1e-3) / 1e12}
    # mixed-precision stack: 2-bit codes in the even layers, the 4-bit layers of the main run in the odd ones
    if layers4 is not None:
        mixed = []
        for l in range(L):
            if l % 2 == 0:
                t = si.layer_tensors(shape, l, 0, device=dev)
                mixed.append(qt.quantize_layer(t, 2, shape.group, keep_canonical=False))
                del t
            else:
                mixed.append(layers4[l])
        mstack = qt.Stack(cfg, mixed)
        qt.qtale_stack_forward(ctx, mstack, xs[0], offs, pos, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            qt.qtale_stack_forward(ctx, mstack, xs[1], offs, pos, workspace=ws)
        torch.cuda.synchronize()
        out["mixed_2_4_bit_prefill_tokens_per_s"] = T * 3 / (time.perf_counter() - t0)
        del mstack, mixed
    del xs, ws
    if not no_decode:
        out["decode"] = decode_section(qt, si, torch, layers, L, bits=3, ratios=(1.0, 0.4), steps=16, graph_steps=0,
                                       label="3-bit codes")["by_exec_ratio"]
    return out


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
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-int3", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the configs[3] (8B GQA) and configs[4] (13B) sections")
    ap.add_argument("--decode-steps", type=int, default=256, help="generated steps per ratio in the configs[2] section")
    ap.add_argument("--no-graph", action="store_true", help="profiling aid: leave the HIP-graph replay leg out of the decode sections")
    ap.add_argument("--decode-only", type=float, default=None, metavar="RATIO",
                    help="profiling aid: run only the decode section at this execution ratio and print its JSON")
    ap.add_argument("--long-attention", action="store_true",
                    help="profiling aid: one layer of the stack on 2 x 4096 tokens at ratio 1.0, prints the prefill attention rate")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (calibrates FETCH_SIZE/WRITE_SIZE under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only: the library runs on a single GPU (run with --gpus 1)")

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
    if args.long_attention:
        Bl, Sl = 2, 4096
        o2, p2 = si.equal_sequences(Bl, Sl)
        o2, p2 = o2.to(dev), p2.to(dev)
        ctx = qt.Context()
        qt.qtale_set_exec_ratio(ctx, 1.0)
        xl = si.hidden_states(shape, Bl * Sl, 0, extra=9000, device=dev)
        for _ in range(2):
            qt.qtale_layer_forward(ctx, cfg, layers[0], xl.clone(), o2, p2)
        xr = [xl.clone() for _ in range(5)]
        qt.qtale_profile_enable(ctx, True)
        torch.cuda.synchronize()
        for xi in xr:
            qt.qtale_layer_forward(ctx, cfg, layers[0], xi, o2, p2)
        prof = qt.qtale_profile_read(ctx)
        a_ms = prof["attention"][0] / prof["attention"][1]
        fl = 4.0 * Sl * Sl / 2 * shape.n_heads * shape.head_dim * Bl
        print(json.dumps({"long_attention": {"workload": "one layer, 2 x 4096 tokens, ratio 1.0, 32 heads x 128", "attention_ms": a_ms,
                                             "attention_TFLOPs_causal": fl / (a_ms * 1e-3) / 1e12}}))
        return
    if args.decode_only is not None:
        print(json.dumps({"decode": decode_section(qt, si, torch, layers, L, ratios=(args.decode_only,), steps=16,
                                                   graph_steps=0 if args.no_graph else 16)}))
        return
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

    if args.traffic_probe:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)       # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

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
    roofline = {"bound": "mfma", "kernel": "qtale::gemm_w4a16_kernel<4,1,4,4,2,1,2,2,false> (gate/up GEMM with SiLU*up epilogue)",
                "achieved": achieved, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_F16_PEAK_TFLOPS, "traffic": recorded_traffic(),
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

    # threshold mode (Eq. 9 with one global theta, data-dependent count kept on the device): calibrate theta
    # for the target ratio on one batch with the two-phase grid search, then time steps at that theta
    threshold = None
    if not args.no_sweep:
        xc = batches(1, 4000)[0]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        theta, r_avg, seen = qt.qtale_calibrate_threshold(ctx, stack, xc, offs, pos, args.ratio, workspace=ws)
        t_cal = time.perf_counter() - t0
        xs = batches(4, 5000)
        cnt = torch.zeros(L, dtype=torch.int32, device=dev)
        qt.qtale_stack_forward(ctx, stack, xs[0], offs, pos, sel_count=cnt, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(xs[1:])
        torch.cuda.synchronize()
        dt_thr = (time.perf_counter() - t0) / 3
        fresh_ratio = float(cnt.sum().item()) / (L * T)
        # like for like: ratio mode at the executed fraction the threshold produced on these batches (the per-layer
        # counts of threshold mode are not multiples of the 128-row tile, ratio 0.5 of 8192 is)
        qt.qtale_set_exec_ratio(ctx, fresh_ratio)
        xs = batches(4, 5000)
        run(xs[:1])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(xs[1:])
        torch.cuda.synchronize()
        dt_same = (time.perf_counter() - t0) / 3
        threshold = {"target_ratio": args.ratio, "theta": theta, "calibration_ratio": r_avg,
                     "candidates_evaluated": len(seen), "calibration_s": t_cal,
                     "fresh_batch_ratio": fresh_ratio,
                     "tokens_per_s": T / dt_thr, "ms_per_step": dt_thr * 1e3,
                     "ratio_mode_at_the_same_executed_fraction_ms_per_step": dt_same * 1e3,
                     "overhead_vs_ratio_mode": dt_thr / dt_same - 1.0}
        qt.qtale_set_exec_ratio(ctx, args.ratio)
    # the same stack with the paper's two-output MLP router (one hidden ReLU layer of 16 units) instead of the
    # linear one
    mlp = None
    if not args.no_sweep:
        mlp_layers = [qt.LayerWeights(lw.lin["q"], lw.lin["k"], lw.lin["v"], lw.lin["o"], lw.lin["gate"], lw.lin["up"],
                                      lw.lin["down"], lw.norm1, lw.norm2, None, 0.0,
                                      si.router_mlp(shape, l, 0, 16, device=dev)) for l, lw in enumerate(layers)]
        mlp_stack = qt.Stack(cfg, mlp_layers)
        xs = batches(4, 6000)
        qt.qtale_stack_forward(ctx, mlp_stack, xs[0], offs, pos, workspace=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for x in xs[1:]:
            qt.qtale_stack_forward(ctx, mlp_stack, x, offs, pos, workspace=ws)
        torch.cuda.synchronize()
        dt_mlp = (time.perf_counter() - t0) / 3
        xs = batches(1, 6100)
        qt.qtale_profile_enable(ctx, True)
        qt.qtale_stack_forward(ctx, mlp_stack, xs[0], offs, pos, workspace=ws)
        prof_mlp = qt.qtale_profile_read(ctx)
        qt.qtale_profile_enable(ctx, False)
        r_ms = prof_mlp["router"][0] / prof_mlp["router"][1]
        mlp = {"router": "two-output MLP, 16 hidden ReLU units, fp64 accumulation", "tokens_per_s": T / dt_mlp,
               "ms_per_step": dt_mlp * 1e3, "router_kernel_ms": r_ms,
               "router_fp64_TFLOPs": 2.0 * T * shape.hidden * 16 / (r_ms * 1e-3) / 1e12}
        del mlp_stack, mlp_layers
    del xs, ws
    # one 1024-token prompt through the same stack: a few hundred executed rows per layer, where the
    # hidden-size-wide linears run on 64-row tiles
    single = None
    if not args.no_sweep:
        S1 = 1024
        o1, p1 = si.equal_sequences(1, S1)
        o1, p1 = o1.to(dev), p1.to(dev)
        ws1 = qt.alloc_workspace(cfg, S1, 1, dev)
        single = {"workload": "same stack, one prompt of %d tokens" % S1, "by_exec_ratio": {}}
        for r in (1.0, 0.5, 0.3):
            qt.qtale_set_exec_ratio(ctx, r)
            xs = [si.hidden_states(shape, S1, 0, extra=7000 + i, device=dev) for i in range(9)]
            qt.qtale_stack_forward(ctx, stack, xs[0], o1, p1, workspace=ws1)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for x in xs[1:]:
                qt.qtale_stack_forward(ctx, stack, x, o1, p1, workspace=ws1)
            torch.cuda.synchronize()
            dt1 = (time.perf_counter() - t0) / 8
            single["by_exec_ratio"]["%.1f" % r] = {"tokens_per_s": S1 / dt1, "ms_per_step": dt1 * 1e3}
        qt.qtale_set_exec_ratio(ctx, args.ratio)
        del xs, ws1
    # what the box itself delivers, for scale: a plain device copy and the vendor library's dense fp16 GEMM of
    # the gate/up shape on random data (neither is part of the path)
    ceilings = None
    if not args.no_sweep:
        src = torch.randn(256 * 1024 * 1024 // 4, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        copy_gbps = 10 * 2 * src.numel() * 4 / (time.perf_counter() - t0) / 1e9
        del src, dst
        a16 = torch.randn(k_exec, H, device=dev, dtype=torch.float16)
        w16 = torch.randn(2 * I, H, device=dev, dtype=torch.float16) * 0.02
        for _ in range(3):
            torch.matmul(a16, w16.t())
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            torch.matmul(a16, w16.t())
        torch.cuda.synchronize()
        lib_tflops = 10 * gu_flops / (time.perf_counter() - t0) / 1e12
        del a16, w16
        ceilings = {"device_copy_256MiB_GBps_read_plus_write": copy_gbps,
                    "vendor_fp16_gemm_same_shape_TFLOPs": lib_tflops,
                    "note": "torch copy_ and torch.matmul (fp16 x fp16, random data) on this GPU, M=%d N=%d K=%d" % (k_exec, 2 * I, H)}
    int3 = None
    if not args.no_int3:
        int3 = int3_section(qt, si, torch, shape, L, B, S, args.ratio, args.no_decode, layers)
    decode = None
    if not args.no_decode:
        gs = 0 if args.no_graph else 32
        decode = decode_section(qt, si, torch, layers, L, steps=args.decode_steps, graph_steps=gs)
        small = decode_section(qt, si, torch, layers, L, B=8, ratios=(1.0, 0.5), steps=32, graph_steps=gs,
                               label="same stack, batch 8")
        decode["batch_8"] = {r: {k: v[k] for k in ("tokens_per_s", "ms_per_step", "hip_graph_ms_per_step", "executed_per_layer")}
                             for r, v in small["by_exec_ratio"].items()}
    # the other workload configurations: LLaMA-3-8B-shaped GQA prefill 4 x 4096 at ratio 0.6, and the LLaMA-13B-shaped
    # stack (prefill 16 x 512, then decode batch 128 on 4096 cached entries) over a sweep of ratios
    others = None
    if not args.no_other_configs:
        del layers, stack
        torch.cuda.empty_cache()
        others = {}
        l8 = quantized_stack(qt, si, torch, si.C4, 32)
        others["configs[3]"] = prefill_section(qt, si, torch, si.C4, l8, 4, 4096, (0.6, 1.0), "configs[3]", steps=2)
        # a call of 32768 tokens: the selection kernel (one workgroup for any T) no longer holds its keys on chip
        # beyond 16384 tokens; its share of a layer at this size, from HIP events over two layers
        long_call = prefill_section(qt, si, torch, si.C4, l8[:2], 8, 4096, (0.6,), "configs[3] shape, 8 x 4096", steps=1)
        ms = long_call["by_exec_ratio"]["0.6"]["kernel_ms_per_launch"]
        others["select_kernel_at_32768_tokens"] = {"workload": long_call["workload"], "select_ms": ms["select"],
                                                   "layer_ms": sum(ms.values()),
                                                   "share_of_layer": ms["select"] / sum(ms.values())}
        del l8
        torch.cuda.empty_cache()
        l13 = quantized_stack(qt, si, torch, si.C5, 40)
        c5 = {"prefill": prefill_section(qt, si, torch, si.C5, l13, 16, 512, (0.5, 0.3, 1.0), "configs[4] prefill", steps=2)}
        if not args.no_decode:
            # 40 layers x 128 sequences x 4096 entries of K and V are 430 GB, more than the 288 GB of HBM: 12 distinct
            # per-layer buffers (129 GB) are shared round-robin by the 40 layers
            c5["decode"] = decode_section(qt, si, torch, l13, 40, B=128, ctx_len=4096, steps=8, ratios=(1.0, 0.5, 0.3),
                                          base=si.C5, kv_distinct=12, graph_steps=0, label="configs[4] decode")
        others["configs[4]"] = c5
        del l13
        torch.cuda.empty_cache()

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
        "threshold_mode": threshold,
        "mlp_router": mlp,
        "single_prompt": single,
        "box_ceilings": ceilings,
        "decode": decode,
        "int3": int3,
        "other_configs": others,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, B, S, args.ratio, L)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
