#!/usr/bin/env python3
"""Benchmark of the MoE verify layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: moe_route_topk -> moe_permute -> moe_expert_up_swiglu_gather -> moe_expert_down ->
moe_combine -> spec_accept.  Prints ONE JSON line: tokens/s of the whole step, the roofline
figure of the gate/up expert GEMM (HIP events around it), and the CPU oracle's rate on a bounded
sample of the same batch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..6] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_FP32_TFLOPS = 157.3       # fp32 vector
PEAK_HBM_GBS = 8000.0          # HBM3E, published


def cpu_baseline(cfg, L, draft, target, budget_s=15.0):
    """The fp64 oracle, as it stands, timed on this machine's host cores on a bounded token sample."""
    import numpy as np
    from oracle import moe_verify_oracle as orc
    from workloads import synth
    try:
        from threadpoolctl import threadpool_info
        blas = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        cores = max(blas) if blas else len(os.sched_getaffinity(0))
    except Exception:
        cores = len(os.sched_getaffinity(0))
    # input preparation (not timed): exact widening of the run-dtype tensors to fp64
    wr = synth.to_f64(L["w_router"])
    bias = None if L["bias"] is None else synth.to_f64(L["bias"])
    wg = [synth.to_f64(L["w_gate"][e]) for e in range(cfg.E)]
    wu = [synth.to_f64(L["w_up"][e]) for e in range(cfg.E)]
    wd = [synth.to_f64(L["w_down"][e]) for e in range(cfg.E)]
    x = synth.to_f64(L["x"])

    def run(n):
        t0 = time.perf_counter()
        orc.moe_layer_stepwise(x[:n], wr, wg, wu, wd, cfg.k, bias, cfg.renorm)
        orc.accept(draft.numpy(), target.numpy())
        return time.perf_counter() - t0

    # bounded sample: the first n tokens of the batch, n chosen from a probe so that the timed
    # run takes roughly budget_s seconds; if the whole batch is faster than that, repeat it
    n0 = min(cfg.T, 64)
    t_probe = run(n0)
    n = int(min(cfg.T, max(n0, n0 * budget_s / max(t_probe, 1e-6))))
    reps, t = 0, 0.0
    while reps == 0 or (t < 0.6 * budget_s and reps < 50):
        t += run(n)
        reps += 1
    return {"value": n * reps / t, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 numpy oracle (route, permute, grouped SwiGLU, combine, accept) on the "
                      f"first {n} of {cfg.T} tokens of the same batch, {reps} pass(es), all "
                      f"{cfg.E} experts' weights widened to fp64 beforehand (untimed); {t:.1f} s"}


def speculation_bench(args):
    """Timings of the speculation-phase / verification-rule kernels (one JSON line):
    affinity table (offline), nearest draft expert, draft routing, sampling-based acceptance,
    greedy head.  Each entry: microseconds per launch, algorithmic bytes, fraction of HBM peak."""
    import torch
    import paper_2604_10152_amd as sm
    from workloads import synth
    sm.load_library()
    torch.cuda.set_device(0)
    I32 = torch.int32
    res = {}

    def timed(name, fn, nbytes, reps=20):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        res[name] = {"us": us, "bytes": nbytes, "hbm_frac": nbytes / (us * 1e-6) / 1e9 / PEAK_HBM_GBS}

    for cid in (2, 3):
        cfg = synth.CONFIGS[cid]
        L = synth.make_layer(cfg, "cuda", seed=args.seed)
        E, d, f = cfg.E, cfg.d_model, cfg.d_ff
        table = torch.empty((E, E), dtype=torch.float32, device="cuda")
        ws = torch.empty((sm.moe_affinity_table_workspace_bytes(E),), dtype=torch.uint8, device="cuda")
        timed(f"affinity_table_cfg{cid}",
              lambda: sm.moe_affinity_table(L["w_gate"], L["w_up"], L["w_down"], table, ws),
              3 * E * d * f * 2, reps=5)
        layer = sm.MoEVerifyLayer(cfg.T, d, f, E, cfg.k, cfg.torch_dtype, renorm=cfg.renorm)
        layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"])
        n_draft = max(cfg.k, E // 4)
        hot = torch.empty((n_draft,), dtype=I32, device="cuda")
        remap = torch.empty((E,), dtype=I32, device="cuda")
        timed(f"hot_experts+nearest_draft_cfg{cid}",
              lambda: (sm.moe_hot_experts(layer.expert_offsets, hot),
                       sm.moe_nearest_draft_expert(table, hot, remap)), E * E * 4)
        T = cfg.B            # the draft model scores one token per sequence and step
        dl = sm.MoEVerifyLayer(T, d, f, E, cfg.k, cfg.torch_dtype, renorm=cfg.renorm)
        xs = L["x"][:T].contiguous()
        timed(f"draft_layer_cfg{cid}_N{n_draft}_T{T}",
              lambda: dl.forward(xs, L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                                 draft_remap=remap), 3 * n_draft * d * f * 2)
        del L, layer, dl
    B, gamma, V = 256, 7, 32000
    g = torch.Generator(device="cuda").manual_seed(args.seed)
    pt = torch.softmax(torch.randn(B, gamma + 1, V, generator=g, device="cuda") * 3, dim=-1)
    pd = torch.softmax(torch.log(pt[:, :gamma]) + 0.7 * torch.randn(B, gamma, V, generator=g, device="cuda"), dim=-1)
    draft = torch.multinomial(pd.reshape(-1, V), 1, generator=g).reshape(B, gamma).to(I32)
    ua = torch.rand(B, gamma, generator=g, device="cuda")
    us = torch.rand(B, generator=g, device="cuda")
    alen = torch.empty((B,), dtype=I32, device="cuda")
    out = torch.empty((B, gamma + 1), dtype=I32, device="cuda")
    timed("spec_accept_sample_B256_g7_V32000",
          lambda: sm.spec_accept_sample(draft, pd.contiguous(), pt, ua, us, alen, out), B * 2 * V * 4)
    logits = torch.randn(B * (gamma + 1), V, generator=g, device="cuda").to(torch.bfloat16)
    tok = torch.empty((B * (gamma + 1),), dtype=I32, device="cuda")
    timed("spec_greedy_tokens_R2048_V32000_bf16", lambda: sm.spec_greedy_tokens(logits, tok),
          B * (gamma + 1) * V * 2)
    print(json.dumps({"metric": "speculation_phase_kernel_us", "data": "synthetic", "n_gpus": 1,
                      "mean_accept_len_sampling": float(alen.float().mean().item()), "kernels": res}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, choices=[1, 2, 3, 4, 5, 6])
    ap.add_argument("--seed", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=["verify", "speculation"], default="verify",
                    help="verify (default): the MoE verify layer, the line the harness reads; "
                         "speculation: per-kernel timings of the draft-routing / sampling rows")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the extra 80-token measurement that the default line carries")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a captured HIP graph (one launch per step); the "
                         "gate/up kernel time for the roofline then comes from an eager pass "
                         "run right after the timed region")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, run one 1 GiB device copy (a kernel of known "
                         "traffic to scale rocprofv3's FETCH_SIZE / WRITE_SIZE against)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_10152_amd as sm
    from workloads import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if args.mode == "speculation":
        speculation_bench(args)
        return
    sm.load_library()
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    stacked = cfg.n_layers > 1
    if stacked:
        x0, layers = synth.make_stack(cfg, "cuda", seed=args.seed)
        L = dict(layers[0], x=x0)
    else:
        L = synth.make_layer(cfg, "cuda", seed=args.seed)
    draft, target = synth.make_tokens(cfg, seed=args.seed)
    draft_d, target_d = draft.cuda(), target.cuda()
    alen = torch.empty(cfg.B, dtype=torch.int32, device="cuda")
    toks = torch.empty(cfg.B, cfg.gamma + 1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    if stacked:
        stack = sm.MoEVerifyStack(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype,
                                  renorm=cfg.renorm)
        layer = stack.layer

        def step(ev=None):
            stack.forward(x0, layers, stream=stream, up_events=ev)
            sm.spec_accept(draft_d, target_d, alen, toks, stream)
    else:
        layer = sm.MoEVerifyLayer(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype,
                                  renorm=cfg.renorm)

        def step(ev=None):
            layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                          stream=stream, up_events=ev)
            sm.spec_accept(draft_d, target_d, alen, toks, stream)

    for _ in range(args.warmup):
        step()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
    if args.graph:
        if stacked:
            graphed = sm.GraphedStep(lambda st: (stack.forward(x0, layers, stream=st),
                                                 sm.spec_accept(draft_d, target_d, alen, toks, st)))
        else:
            graphed = sm.GraphedStep(lambda st: (
                layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                              stream=st),
                sm.spec_accept(draft_d, target_d, alen, toks, st)))
        for _ in range(max(1, args.warmup // 2)):
            graphed.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphed.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(args.steps):            # kernel time for the roofline: eager, untimed
            step(events[i])
        torch.cuda.synchronize()
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(events[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    up_ms = sum(a.elapsed_time(b) for a, b in events) / args.steps

    counts = (layer.expert_offsets[1:] - layer.expert_offsets[:-1]).cpu()
    active = int((counts > 0).sum())
    esize = 4 if cfg.dtype == "f32" else 2
    P, d, f = cfg.P, cfg.d_model, cfg.d_ff
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)
    tflops = cfg.flops() * cfg.n_layers / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the gate/up expert GEMM with the SwiGLU epilogue (2/3 of the flops)
    up_flops = 4.0 * P * d * f
    # bytes: the active experts' two matrices once, every x row once (the gather re-reads hit
    # the cache), h once
    up_bytes = (active * 2 * d * f + cfg.T * d + P * f) * esize
    if cfg.dtype == "bf16" and args.config == 4:
        roof = {"bound": "mfma", "achieved": up_flops / (up_ms * 1e-3) / 1e12,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
    elif cfg.dtype == "bf16":
        roof = {"bound": "hbm", "achieved": up_bytes / (up_ms * 1e-3) / 1e9,
                "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "alu", "achieved": up_flops / (up_ms * 1e-3) / 1e12,
                "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if cfg.dtype != "bf16":
        roof["kernel"] = "grouped_gemm_f32_kernel<true> (gate/up + SwiGLU)"
    elif args.config == 4:
        roof["kernel"] = "grouped_gemm_bf16_pipe16_kernel<PipeCfg<320,256,32,4,2,4,true>> (gate/up + SwiGLU)"
    elif d >= 4096:
        roof["kernel"] = "grouped_gemm_bf16_pipe_kernel<PipeCfg<64,128,64,4,1,2,true>> (gate/up + SwiGLU)"
    else:
        roof["kernel"] = "grouped_gemm_bf16_kernel<TileCfg<64,256,1,4,true>> (gate/up + SwiGLU)"
    roof["kernel_ms"] = up_ms
    roof["traffic"] = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            roof["traffic"] = json.load(open(tpath)).get(f"cfg{args.config}")
        except Exception:
            roof["traffic"] = None

    out = {
        "metric": "expert_layer_tokens_per_s", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "gamma": cfg.gamma, "tokens": cfg.T,
                   "d_model": d, "d_ff": f, "experts": cfg.E, "top_k": cfg.k,
                   "active_experts": active, "max_rows_per_expert": int(counts.max())},
        "launch": "hip-graph" if args.graph else "eager",
        "tflops": tflops, "mfma_frac": tflops / PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else None,
        "roofline": roof,
    }
    if args.config == 4 and not args.graph and not args.no_also:
        # same weights, the 80-token batch of the Mixtral-shaped configuration (B=16, gamma=4):
        # the memory-bound end of the same layer, reported beside the headline workload
        c2 = synth.CONFIGS[2]
        x2 = L["x"][:c2.T].contiguous()
        lay2 = sm.MoEVerifyLayer(c2.T, d, f, cfg.E, cfg.k, cfg.torch_dtype, renorm=cfg.renorm)
        d2, t2 = synth.make_tokens(c2, seed=args.seed)
        d2, t2 = d2.cuda(), t2.cuda()
        al2 = torch.empty(c2.B, dtype=torch.int32, device="cuda")
        tk2 = torch.empty(c2.B, c2.gamma + 1, dtype=torch.int32, device="cuda")
        ev2 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(args.steps)]

        def step2(ev=None):
            lay2.forward(x2, L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                         stream=stream, up_events=ev)
            sm.spec_accept(d2, t2, al2, tk2, stream)

        for _ in range(args.warmup):
            step2()
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for i in range(args.steps):
            step2(ev2[i])
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - ta) * 1e3 / args.steps
        up2 = sum(a.elapsed_time(b) for a, b in ev2) / args.steps
        act2 = int(((lay2.expert_offsets[1:] - lay2.expert_offsets[:-1]) > 0).sum())
        bytes2 = (act2 * 2 * d * f + c2.T * d + c2.P * f) * esize
        out["also"] = {c2.name: {
            "tokens": c2.T, "ms_per_step": ms2, "tokens_per_s": c2.T / (ms2 * 1e-3),
            "tflops": c2.flops() / (ms2 * 1e-3) / 1e12,
            "roofline": {"bound": "hbm", "achieved": bytes2 / (up2 * 1e-3) / 1e9,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": bytes2 / (up2 * 1e-3) / 1e9 / PEAK_HBM_GBS,
                         "kernel": "grouped_gemm_bf16_pipe_kernel<PipeCfg<64,128,64,4,1,2,true>> "
                                   "(gate/up + SwiGLU)", "kernel_ms": up2}}}
    if stacked:
        out["config"]["layers"] = cfg.n_layers
        out["accepted_tokens_per_s"] = float(alen.sum().item()) / (ms_per_step * 1e-3)
        out["mean_accept_len"] = float(alen.float().mean().item())
        args.no_cpu_baseline = True      # the bounded oracle sample is defined for one layer
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()   # evicts src
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst, flush
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, L, draft, target)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
