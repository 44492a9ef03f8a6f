#!/usr/bin/env python3
"""Benchmark of the MoE verify layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: moe_route_topk -> moe_permute -> moe_expert_up_swiglu_gather -> moe_expert_down ->
moe_combine -> spec_accept.  Prints ONE JSON line: tokens/s of the whole step, the per-kernel
split (HIP events on the launch stream, medians over the timed steps) with both roofline
fractions of the two expert GEMMs, the same for the other configurations (`also`), the paper's
own quantities measured on this layer (lambda, c and the Eq. 2 estimate), and the CPU oracle's
rate on a bounded sample of the same batch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..6] [--no-cpu-baseline]
    python bench.py --mode peaks          measured ceilings of this machine (MFMA, HBM, L2 -> LDS)
    python bench.py --mode speculation    speculation-phase / verification-rule kernels
    python bench.py --mode traffic        short run to collect HBM traffic counters under rocprofv3
    python bench.py --mode traffic-report <pmc csv> ...   turns those counters into profiles/traffic.json
"""
import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_FP32_TFLOPS = 157.3       # fp32 vector
PEAK_HBM_GBS = 8000.0          # HBM3E, published
SETTLE_MS = 60.0               # untimed load before the warm-up steps (see LayerRun.settle)


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


PAPER_CONTEXT = {       # the paper's own figures, other hardware: context only, never a target
    "throughput_speedup_max": 4.30, "hardware": "H100 96 GB + host DRAM over PCIe 5.0 (expert offloading)",
    "lambda_B1_gamma8": 6.0, "lambda_B32": 2.0, "cite": "Sec. 3.3; abstract"}


def speculative_speedup(tau, gamma, c, lam=1.0):
    """Eq. 2 of the paper: S = tau / (gamma * c + lambda); lambda = 1 gives Eq. 1."""
    return float(tau) / (float(gamma) * float(c) + float(lam))


def source_fingerprint():
    """sha256 over the kernel sources: ties a stored counter figure to the build it was taken on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2604_10152_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


KERNELS = ("route", "permute", "up", "down", "combine", "accept")


def algorithmic_work(cfg, T, active, rows_materialised=False):
    """Flops and bytes every kernel of one layer has to do at T tokens (algorithmic: the
    active experts' weights once, activations and intermediates read and written once).
    rows_materialised: the permute step writes the dispatched token rows (tile-packed path);
    otherwise the gate/up kernel gathers them from the token matrix itself."""
    es = 4 if cfg.dtype == "f32" else 2
    d, f, E, k = cfg.d_model, cfg.d_ff, cfg.E, cfg.k
    P = T * k
    moved = (T * d + P * d) * es if rows_materialised else 0
    x_read = P * d if rows_materialised else T * d
    return {
        "route": {"flops": 2.0 * T * d * E, "bytes": (T * d + E * d) * es + P * 8},
        "permute": {"flops": 0.0, "bytes": P * 4 * 3 + (E + 1) * 4 + moved},
        "up": {"flops": 4.0 * P * d * f, "bytes": (active * 2 * d * f + x_read + P * f) * es},
        "down": {"flops": 2.0 * P * d * f, "bytes": (active * d * f + P * f + P * d) * es},
        "combine": {"flops": 2.0 * P * d, "bytes": (P * d + T * d) * es + P * 8},
        "accept": {"flops": 0.0, "bytes": cfg.B * (2 * cfg.gamma + 2) * 4 * 2},
    }


class LayerRun:
    """One layer configuration set up for timing: buffers, token ids, the step closure."""

    def __init__(self, torch, sm, synth, cfg, L, T=None, B=None, gamma=None, seed=0, draft_remap=None,
                 packed=None):
        self.torch, self.sm, self.cfg, self.L = torch, sm, cfg, L
        self.T = cfg.T if T is None else T
        self.B = cfg.B if B is None else B
        self.gamma = cfg.gamma if gamma is None else gamma
        self.x = L["x"][:self.T].contiguous()
        self.layer = sm.MoEVerifyLayer(self.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype,
                                       renorm=cfg.renorm)
        draft, target = synth.make_tokens(cfg, seed=seed, B=self.B, gamma=self.gamma)
        self.draft, self.target = draft, target
        self.draft_d, self.target_d = draft.cuda(), target.cuda()
        self.alen = torch.empty(self.B, dtype=torch.int32, device="cuda")
        self.toks = torch.empty(self.B, self.gamma + 1, dtype=torch.int32, device="cuda")
        self.stream = torch.cuda.current_stream()
        self.draft_remap = draft_remap
        self.packed = packed      # tile-packed expert weights (the layer decides where to use them)

    def step(self, marks=None):
        L = self.L
        self.layer.forward(self.x, L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                           stream=self.stream, marks=marks, draft_remap=self.draft_remap,
                           packed=self.packed)
        self.sm.spec_accept(self.draft_d, self.target_d, self.alen, self.toks, self.stream)
        if marks is not None:
            marks[6].record(self.stream)

    def settle(self, ms=SETTLE_MS):
        """Untimed steps for about `ms` of wall time before the warm-up: a chip that comes out of
        idle starts at its highest clock, then the power controller overshoots downwards (the
        large-batch gate/up kernel: 740, 820, 1130, 1040, 960, 910 us ... on consecutive
        launches) and takes 15-20 ms of load to settle (770-800 us from then on, flat over
        hundreds of steps).  The timed region measures that steady state."""
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(4):
                self.step()
            self.torch.cuda.synchronize()

    def measure(self, steps, warmup, back_to_back=True):
        """W untimed steps, then the timed region: exactly K steps between two synchronisations,
        seven HIP events per step on the launch stream (per-kernel times, per-step medians).
        Every event between two kernels puts a marker packet between them (about 6 us of idle
        stream each, 40 us per step), so a second pass of K steps with nothing but the step's
        own launches on the stream is timed as well (`ms_per_step_back_to_back`: wall clock, and
        the median over five groups of consecutive steps from boundary events).  The two differ
        by 1-2 % either way at the benchmark workload: the chip runs at its power limit, and the
        idle gaps of the instrumented pass are paid back by a higher clock inside the kernels."""
        torch = self.torch
        self.settle()
        for _ in range(warmup):
            self.step()
        marks = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(marks[i])
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        b2b_ms = b2b_median = None
        if back_to_back:
            n_groups = min(5, steps)
            edges = [round(g * steps / n_groups) for g in range(n_groups + 1)]
            bounds = [torch.cuda.Event(enable_timing=True) for _ in edges]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g = 0
            for i in range(steps):
                if i == edges[g]:
                    bounds[g].record(self.stream)
                    g += 1
                self.step()
            bounds[-1].record(self.stream)
            torch.cuda.synchronize()
            b2b_ms = (time.perf_counter() - t0) * 1e3 / steps
            b2b_median = statistics.median(
                bounds[g].elapsed_time(bounds[g + 1]) / (edges[g + 1] - edges[g])
                for g in range(n_groups))
        per = {n: [] for n in KERNELS}
        whole = []
        for m in marks:
            for j, n in enumerate(KERNELS):
                per[n].append(m[j].elapsed_time(m[j + 1]))
            whole.append(m[0].elapsed_time(m[6]))
        counts = (self.layer.expert_offsets[1:] - self.layer.expert_offsets[:-1]).cpu()
        active = int((counts > 0).sum())
        packed_rows = (self.packed is not None and self.cfg.dtype == "bf16" and
                       self.layer.packed_plan(self.T * self.cfg.k, self.cfg.E, self.cfg.d_model,
                                              self.cfg.d_ff)[0])
        work = algorithmic_work(self.cfg, self.T, active, rows_materialised=packed_rows)
        kernels = {}
        for n in KERNELS:
            ms = statistics.median(per[n])
            w = work[n]
            e = {"us": ms * 1e3, "us_mean": statistics.fmean(per[n]) * 1e3, "bytes": w["bytes"],
                 "gbs": w["bytes"] / (ms * 1e-3) / 1e9,
                 "hbm_frac": w["bytes"] / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
            if n in ("up", "down"):
                e["flops"] = w["flops"]
                e["tflops"] = w["flops"] / (ms * 1e-3) / 1e12
                e["mfma_frac"] = e["tflops"] / (PEAK_BF16_TFLOPS if self.cfg.dtype == "bf16"
                                                else PEAK_FP32_TFLOPS)
                e["us_min"], e["us_max"] = min(per[n]) * 1e3, max(per[n]) * 1e3
            kernels[n] = e
        return {"ms_per_step": wall_ms, "ms_per_step_median": statistics.median(whole),
                "ms_per_step_back_to_back": b2b_ms, "ms_per_step_back_to_back_median": b2b_median,
                "kernels": kernels, "active_experts": active, "packed_up": bool(packed_rows),
                "max_rows_per_expert": int(counts.max()), "min_rows_per_expert": int(counts.min())}


def packed_weights_for(sm, torch, cfg, L, T, row_major=False):
    """Tile-packed copies of the expert weights if the layer runs any projection of a T-token
    batch on them (one-time re-layout, outside every timed region: the weights are resident model
    parameters); None otherwise."""
    if cfg.dtype != "bf16" or row_major:
        return None
    if not sm.MoEVerifyLayer.packed_plan(T * cfg.k, cfg.E, cfg.d_model, cfg.d_ff)[0]:
        return None
    packed = sm.MoEVerifyLayer.pack_weights(L["w_gate"], L["w_up"], L["w_down"])
    torch.cuda.synchronize()
    return packed


def kernel_name(cfg, T, packed=True):
    """Which gate/up kernel runs for this shape (names for the report)."""
    import paper_2604_10152_amd as sm
    if cfg.dtype != "bf16":
        return "grouped_gemm_f32_kernel<true> (gate/up + SwiGLU)"
    rows = T * cfg.k
    tile = 320 if rows >= 192 * cfg.E else 192
    if packed and sm.MoEVerifyLayer.packed_plan(rows, cfg.E, cfg.d_model, cfg.d_ff)[0]:
        return (f"grouped_gemm_bf16_pipe16_kernel<PipeCfg<{tile},256,32,4,2,4,true>,PA,PB> (gate/up + "
                "SwiGLU on tile-packed operands: the permute step writes the dispatched rows "
                "tile-packed)")
    if rows >= 192 * cfg.E or (cfg.d_model >= 4096 and rows >= 48 * cfg.E):
        return f"grouped_gemm_bf16_pipe16_kernel<PipeCfg<{tile},256,32,4,2,4,true>> (gate/up + SwiGLU)"
    if cfg.d_model >= 4096:
        return "grouped_gemm_bf16_pipe_kernel<PipeCfg<64,128,64,4,1,2,true>> (gate/up + SwiGLU)"
    return "grouped_gemm_bf16_kernel<TileCfg<64,256,1,4,true>> (gate/up + SwiGLU)"


def roofline_of(cfg, T, m, mfma_bound):
    """Roofline entry of the gate/up kernel: algorithmic flops (or bytes) per launch over the
    AVERAGE launch duration of the timed region (HIP events); the median-based fraction beside it."""
    up = m["kernels"]["up"]
    mean_s, med_s = up["us_mean"] * 1e-6, up["us"] * 1e-6
    if cfg.dtype != "bf16" or mfma_bound:
        peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
        r = {"bound": "mfma" if cfg.dtype == "bf16" else "alu", "achieved": up["flops"] / mean_s / 1e12,
             "peak": peak, "unit": "TFLOP/s", "frac_median": up["flops"] / med_s / 1e12 / peak}
    else:
        r = {"bound": "hbm", "achieved": up["bytes"] / mean_s / 1e9, "peak": PEAK_HBM_GBS,
             "unit": "GB/s", "frac_median": up["bytes"] / med_s / 1e9 / PEAK_HBM_GBS}
    r["frac"] = r["achieved"] / r["peak"]
    r["kernel"] = kernel_name(cfg, T, packed=m.get("packed_up", False))
    r["kernel_ms"] = up["us_mean"] * 1e-3
    r["kernel_ms_median"] = up["us"] * 1e-3
    r["traffic"] = None
    return r


def stored_traffic(config_id):
    """HBM bytes per launch of the gate/up kernel from profiles/traffic.json, but only if that
    file was written for exactly this build of the kernels; otherwise None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        t = json.load(open(path))
        if t.get("source_fingerprint") != source_fingerprint():
            return None
        return t.get(f"cfg{config_id}", {}).get("up_bytes")
    except Exception:
        return None


def summary(cfg, T, m):
    """Compact entry of the `also` block for one configuration."""
    ms = m["ms_per_step"]
    flops = 6.0 * T * cfg.k * cfg.d_model * cfg.d_ff + 2.0 * T * cfg.d_model * cfg.E
    return {"tokens": T, "ms_per_step": ms, "ms_per_step_median": m["ms_per_step_median"],
            "ms_per_step_back_to_back": m["ms_per_step_back_to_back"],
            "ms_per_step_back_to_back_median": m["ms_per_step_back_to_back_median"],
            "tokens_per_s": T / (ms * 1e-3), "tflops": flops / (ms * 1e-3) / 1e12,
            "active_experts": m["active_experts"], "max_rows_per_expert": m["max_rows_per_expert"],
            "kernels_us": {n: round(m["kernels"][n]["us"], 2) for n in KERNELS},
            "up": {k: m["kernels"]["up"][k] for k in ("tflops", "mfma_frac", "gbs", "hbm_frac")},
            "down": {k: m["kernels"]["down"][k] for k in ("tflops", "mfma_frac", "gbs", "hbm_frac")},
            "roofline": roofline_of(cfg, T, m, mfma_bound=False)}


def paper_quantities(torch, sm, synth, cfg, L, B, gamma, steps, warmup, seed, t_verify_ms=None,
                     packed=None):
    """lambda, c and the Eq. 2 estimate for this layer at batch size B and draft length gamma
    (Sec. 3.3): lambda = T<B*(gamma+1)> / T<B> on the same weights, c = T_draft<B> / T_target<B>
    with the draft model = the same layer restricted to the E/4 most activated experts of the
    verification pass (nearest-expert substitution), tau = mean generated tokens per step of the
    synthetic ids (per-position match probability 0.7)."""
    import dataclasses
    E, k = cfg.E, cfg.k
    if t_verify_ms is None:
        ver = LayerRun(torch, sm, synth, cfg, L, T=B * (gamma + 1), B=B, gamma=gamma, seed=seed,
                       packed=packed)
        t_verify_ms = ver.measure(steps, warmup)["ms_per_step_back_to_back_median"]
        offsets = ver.layer.expert_offsets
    else:
        ver = LayerRun(torch, sm, synth, cfg, L, T=B * (gamma + 1), B=B, gamma=gamma, seed=seed,
                       packed=packed)
        ver.step()
        offsets = ver.layer.expert_offsets
    tgt = LayerRun(torch, sm, synth, cfg, L, T=B, B=B, gamma=gamma, seed=seed, packed=packed)
    t_target_ms = tgt.measure(steps, warmup)["ms_per_step_back_to_back_median"]
    n_draft = max(k, E // 4)
    table = torch.empty((E, E), dtype=torch.float32, device="cuda")
    ws = torch.empty((sm.moe_affinity_table_workspace_bytes(E),), dtype=torch.uint8, device="cuda")
    sm.moe_affinity_table(L["w_gate"], L["w_up"], L["w_down"], table, ws)
    hot = torch.empty((n_draft,), dtype=torch.int32, device="cuda")
    remap = torch.empty((E,), dtype=torch.int32, device="cuda")
    sm.moe_hot_experts(offsets, hot)
    sm.moe_nearest_draft_expert(table, hot, remap)
    drf = LayerRun(torch, sm, synth, cfg, L, T=B, B=B, gamma=gamma, seed=seed, draft_remap=remap,
                   packed=packed)
    t_draft_ms = drf.measure(steps, warmup)["ms_per_step_back_to_back_median"]
    # tau: synthetic acceptance with match probability 0.7 through spec_accept
    ids_cfg = dataclasses.replace(cfg, match_prob=0.7)
    d_ids, t_ids = synth.make_tokens(ids_cfg, seed=seed, B=max(B, 4096), gamma=gamma)
    alen = torch.empty(d_ids.shape[0], dtype=torch.int32, device="cuda")
    toks = torch.empty(d_ids.shape[0], gamma + 1, dtype=torch.int32, device="cuda")
    sm.spec_accept(d_ids.cuda(), t_ids.cuda(), alen, toks)
    tau = float(alen.float().mean().item())
    lam, c = t_verify_ms / t_target_ms, t_draft_ms / t_target_ms
    return {"B": B, "gamma": gamma, "tokens_verified": B * (gamma + 1), "draft_experts": n_draft,
            "T_target_B_ms": t_target_ms, "T_verify_ms": t_verify_ms, "T_draft_B_ms": t_draft_ms,
            "lambda": lam, "c": c, "tau_synthetic_p0.7": tau,
            "S_eq2": speculative_speedup(tau, gamma, c, lam),
            "S_eq1_lambda_1": speculative_speedup(tau, gamma, c, 1.0)}


def peaks_bench(args):
    """Measured ceilings of this machine, one JSON line each, the published peak beside them."""
    import torch
    from paper_2604_10152_amd import peaks
    torch.cuda.set_device(0)
    st = torch.cuda.current_stream()
    out = torch.empty(2048 * 512, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(2, dtype=torch.int64, device="cuda")

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            r = fn()
            e1.record(st)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = (ms, r) if best is None or ms < best[0] else best
        return best

    for kind, name in ((0, "v_mfma_f32_16x16x32_bf16"), (1, "v_mfma_f32_32x32x16_bf16")):
        for blocks in (256, 512):
            ms, flops = timed(lambda: peaks.mfma(kind, blocks, 20000, out, clocks, st))
            c = clocks.cpu().tolist()
            print(json.dumps({"peak": "mfma_bf16_registers_only", "instruction": name,
                              "workgroups": blocks, "waves_per_simd": 2, "operands": "pseudo-random, "
                              "12 distinct fragments cycled every instruction",
                              "ms": ms, "measured_tflops": flops / ms / 1e9,
                              "published_tflops": PEAK_BF16_TFLOPS,
                              "frac_of_published": flops / ms / 1e9 / PEAK_BF16_TFLOPS,
                              "shader_clock_mhz_under_load": c[0] / max(c[1], 1) * 100.0}), flush=True)
    lsink = torch.zeros(512 * 16, dtype=torch.uint8, device="cuda")
    names = ("consecutive 16-byte pieces",
             "expert GEMM fragment read: 16 rows of 64 bytes, chunk ^ ((row/2)%4)",
             "all lanes in the same banks",
             "same fragment read with chunk ^ ((row/4)%4)")
    for pattern in range(4):
        peaks.lds_read(pattern, 2000, clocks, lsink, st)
        torch.cuda.synchronize()
        c = clocks.cpu().tolist()[0]
        print(json.dumps({"peak": "lds_ds_read_b128", "pattern": names[pattern],
                          "clk_per_wave_instruction_per_cu": c / (2000 * 64),
                          "bytes_per_clk_per_cu": 1024.0 * 2000 * 64 / c}), flush=True)
    buf = torch.zeros(4 << 30, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    for blocks in (2048, 8192):
        ms, nbytes = timed(lambda: peaks.hbm_read(buf, blocks, sink, st))
        print(json.dumps({"peak": "hbm_read_stream", "buffer_bytes": nbytes, "workgroups": blocks,
                          "ms": ms, "measured_gbs": nbytes / ms / 1e6, "published_gbs": PEAK_HBM_GBS,
                          "frac_of_published": nbytes / ms / 1e6 / PEAK_HBM_GBS}), flush=True)
    for seg in (1024, 128, 64):
        for region in (16 << 20, 4 << 30):
            # L2: 1024 workgroups sweep windows inside 16 MB 200 times; HBM: 16384 workgroups
            # read their own 256 KB window of a 4 GiB buffer exactly once
            l2 = region <= (64 << 20)
            blocks, iters = (1024, 200) if l2 else (region // (256 << 10), 1)
            ms, nbytes = timed(lambda: peaks.l2_lds(buf, region, blocks, iters, seg, st))
            print(json.dumps({"peak": "global_load_lds_dwordx4_stream",
                              "source": "L2-resident windows" if l2 else "HBM (4 GiB read once)",
                              "contiguous_bytes_per_row_piece": seg, "workgroups": blocks, "ms": ms,
                              "bytes": nbytes, "measured_gbs": nbytes / ms / 1e6,
                              "published_hbm_gbs": PEAK_HBM_GBS}), flush=True)
    # the same stream out of HBM with the non-temporal hint (what the expert GEMMs use for
    # weight tiles that no other workgroup reads)
    region = 4 << 30
    ms, nbytes = timed(lambda: peaks.l2_lds_nt(buf, region, region // (256 << 10), 1, st))
    print(json.dumps({"peak": "global_load_lds_dwordx4_stream",
                      "source": "HBM (4 GiB read once), non-temporal hint",
                      "contiguous_bytes_per_row_piece": 1024, "workgroups": region // (256 << 10),
                      "ms": ms, "bytes": nbytes, "measured_gbs": nbytes / ms / 1e6,
                      "published_hbm_gbs": PEAK_HBM_GBS}), flush=True)


def traffic_run(args):
    """What rocprofv3 --pmc is pointed at: two calibration launches of known traffic (a 2 GiB
    read-only stream with ordinary loads, a 2 GiB global->LDS stream with the expert GEMMs' own
    load instruction) and three steps of the benchmark workload."""
    import torch
    import paper_2604_10152_amd as sm
    from paper_2604_10152_amd import peaks
    from workloads import synth
    torch.cuda.set_device(0)
    st = torch.cuda.current_stream()
    buf = torch.zeros(2 << 30, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    flush = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
    flush.add_(1)                                                   # pushes buf out of the caches
    peaks.hbm_read(buf, 8192, sink, st)
    flush.add_(1)
    peaks.l2_lds(buf, 2 << 30, 8192, 1, 128, st)                    # 8192 windows of 256 KB: 2 GiB, each byte once
    torch.cuda.synchronize()
    cfg = synth.CONFIGS[args.config]
    L = synth.make_layer(cfg, "cuda", seed=args.seed)
    packed = packed_weights_for(sm, torch, cfg, L, cfg.T, args.row_major)
    run = LayerRun(torch, sm, synth, cfg, L, seed=args.seed, packed=packed)
    for _ in range(3):
        run.step()
    torch.cuda.synchronize()
    print(json.dumps({"mode": "traffic", "config": args.config, "calibration_bytes": 2 << 30,
                      "source_fingerprint": source_fingerprint()}))


def traffic_report(args):
    """Reads rocprofv3 counter CSVs (TCC_EA0_RDREQ_sum, TCC_EA0_RDREQ_32B_sum,
    TCC_EA0_RDREQ_128B_sum in one run; TCC_EA0_WRREQ_sum, TCC_EA0_WRREQ_64B_sum in another) of
    `--mode traffic` and writes profiles/traffic.json: bytes per launch of the expert GEMMs,
    each scaled by what the same counters read for the calibration launch of known size."""
    import csv
    import collections
    vals = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in args.csv:
        for r in csv.DictReader(open(path)):
            vals[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))

    def mean(kname_part, counter, extra=None):
        for k, d in vals.items():
            if kname_part in k and (extra is None or extra in k) and counter in d:
                return sum(d[counter]) / len(d[counter])
        return None

    def read_bytes(part, extra=None):
        rd, r32, r128 = (mean(part, c, extra) for c in
                         ("TCC_EA0_RDREQ_sum", "TCC_EA0_RDREQ_32B_sum", "TCC_EA0_RDREQ_128B_sum"))
        if rd is None:
            return None
        return 128.0 * r128 + 32.0 * r32 + 64.0 * (rd - r128 - r32)

    def write_bytes(part, extra=None):
        wr, w64 = (mean(part, c, extra) for c in ("TCC_EA0_WRREQ_sum", "TCC_EA0_WRREQ_64B_sum"))
        if wr is None:
            return None
        return 64.0 * w64 + 32.0 * (wr - w64)

    known = float(2 << 30)
    cal_plain, cal_dma = read_bytes("hbm_read_loop"), read_bytes("l2_lds_loop")
    out = {"source_fingerprint": source_fingerprint(),
           "calibration": {"known_bytes": known, "plain_load_stream_read": cal_plain,
                           "lds_dma_stream_read": cal_dma,
                           "factor_plain": cal_plain / known if cal_plain else None,
                           "factor_lds_dma": cal_dma / known if cal_dma else None}}
    fac = (cal_dma / known) if cal_dma else 1.0
    entry = {}
    for tag, extra in (("up", "Lb1E"), ("down", "Lb0E")):
        rb, wb = read_bytes("grouped_gemm_bf16", extra), write_bytes("grouped_gemm_bf16", extra)
        entry[f"{tag}_read_bytes"] = rb / fac if rb is not None else None
        entry[f"{tag}_write_bytes"] = wb
        entry[f"{tag}_bytes"] = (rb / fac if rb is not None else 0.0) + (wb or 0.0)
    out[f"cfg{args.config}"] = entry
    path = os.path.join(ROOT, "profiles", "traffic.json")
    json.dump(out, open(path, "w"), indent=1)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, choices=[1, 2, 3, 4, 5, 6])
    ap.add_argument("--seed", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-back-to-back", action="store_true",
                    help="skip the second (event-free) pass: every launch of the run is then one "
                         "of the warm-up or of the timed region (for kernel traces)")
    ap.add_argument("--mode", choices=["verify", "speculation", "peaks", "traffic", "traffic-report"],
                    default="verify",
                    help="verify (default): the MoE verify layer, the line the harness reads; "
                         "speculation: per-kernel timings of the draft-routing / sampling rows; "
                         "peaks: measured MFMA / HBM / L2->LDS ceilings of this box; traffic: the "
                         "short run rocprofv3 --pmc is pointed at; traffic-report: summarises its CSVs")
    ap.add_argument("csv", nargs="*", help="counter CSV files (traffic-report only)")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the other configurations and the paper's quantities (main line only)")
    ap.add_argument("--row-major", action="store_true",
                    help="keep the expert weights row-major for the large-batch workload too "
                         "(default: tile-packed once before the timed region)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a captured HIP graph (one launch per step); the "
                         "per-kernel times then come from an eager pass after the timed region")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.mode == "traffic-report":
        traffic_report(args)
        return

    import torch
    import paper_2604_10152_amd as sm
    from workloads import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    sm.load_library()
    torch.cuda.set_device(0)
    if args.mode == "speculation":
        speculation_bench(args)
        return
    if args.mode == "peaks":
        peaks_bench(args)
        return
    if args.mode == "traffic":
        traffic_run(args)
        return
    cfg = synth.CONFIGS[args.config]
    if cfg.n_layers > 1:
        out = stack_bench(torch, sm, synth, cfg, args)
        print(json.dumps(out))
        return
    L = synth.make_layer(cfg, "cuda", seed=args.seed)
    packed = packed_weights_for(sm, torch, cfg, L, cfg.T, args.row_major)
    run = LayerRun(torch, sm, synth, cfg, L, seed=args.seed, packed=packed)
    if args.graph:
        graphed = sm.GraphedStep(lambda st: (
            run.layer.forward(run.x, L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                              stream=st, packed=packed),
            sm.spec_accept(run.draft_d, run.target_d, run.alen, run.toks, st)))
        run.settle()
        for _ in range(args.warmup):
            graphed.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graphed.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    m = run.measure(args.steps, args.warmup, back_to_back=not args.no_back_to_back)
    ms_per_step = graph_ms if args.graph else m["ms_per_step"]
    d, f = cfg.d_model, cfg.d_ff
    flops = cfg.flops()
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    mfma_bound = cfg.dtype == "bf16" and args.config == 4
    roof = roofline_of(cfg, cfg.T, m, mfma_bound)
    roof["traffic"] = stored_traffic(args.config)
    hbm_bytes = sum(m["kernels"][n]["bytes"] for n in KERNELS)
    out = {
        "metric": "expert_layer_tokens_per_s", "value": cfg.T / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_ms": SETTLE_MS,
        "ms_per_step": ms_per_step, "ms_per_step_median": m["ms_per_step_median"],
        "tokens_per_s_median": cfg.T / (m["ms_per_step_median"] * 1e-3),
        "ms_per_step_back_to_back": m["ms_per_step_back_to_back"],
        "ms_per_step_back_to_back_median": m["ms_per_step_back_to_back_median"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "gamma": cfg.gamma, "tokens": cfg.T,
                   "d_model": d, "d_ff": f, "experts": cfg.E, "top_k": cfg.k,
                   "active_experts": m["active_experts"],
                   "max_rows_per_expert": m["max_rows_per_expert"],
                   "min_rows_per_expert": m["min_rows_per_expert"],
                   "expert_weight_layout": "tile-packed copies next to the row-major weights "
                                           "(moe_pack_weights, once, outside the timed region)"
                                           if packed is not None else "row-major"},
        "launch": "hip-graph" if args.graph else "eager",
        "tflops": tflops, "mfma_frac": tflops / PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else None,
        "hbm_frac": hbm_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "roofline": roof,
        "kernels": m["kernels"],
        "paper_context": PAPER_CONTEXT,
    }
    if args.config == 4 and not args.graph and not args.no_also:
        also = {}
        steps2 = max(10, args.steps // 2)
        # same weights, the 80-token batch of the Mixtral-shaped configuration (B=16, gamma=4):
        # the memory-bound end of the same layer
        c2 = synth.CONFIGS[2]
        r2 = LayerRun(torch, sm, synth, c2, L, seed=args.seed, packed=packed)
        also[c2.name] = summary(c2, c2.T, r2.measure(steps2, args.warmup))
        out["paper_quantities"] = [
            paper_quantities(torch, sm, synth, c2, L, c2.B, c2.gamma, steps2, 5, args.seed,
                             t_verify_ms=also[c2.name]["ms_per_step_back_to_back_median"],
                             packed=packed),
            paper_quantities(torch, sm, synth, cfg, L, cfg.B, cfg.gamma, steps2, 5, args.seed,
                             t_verify_ms=m["ms_per_step_back_to_back_median"], packed=packed),
        ]
        del r2
        for cid in (3, 6):
            cc = synth.CONFIGS[cid]
            Lc = synth.make_layer(cc, "cuda", seed=cid)
            pc = packed_weights_for(sm, torch, cc, Lc, cc.T, args.row_major)
            rc = LayerRun(torch, sm, synth, cc, Lc, seed=cid, packed=pc)
            also[cc.name] = summary(cc, cc.T, rc.measure(steps2, args.warmup))
            also[cc.name]["expert_weight_layout"] = "tile-packed" if pc is not None else "row-major"
            del Lc, rc, pc
            torch.cuda.empty_cache()
        out["also"] = also
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, L, run.draft, run.target)
    if args.config == 4 and not args.graph and not args.no_also:
        del L, run
        torch.cuda.empty_cache()
        c5 = synth.CONFIGS[5]
        s5 = stack_bench(torch, sm, synth, c5, argparse.Namespace(steps=10, warmup=3, seed=5, graph=False))
        out["also"][c5.name] = {k: s5[k] for k in ("ms_per_step", "ms_per_step_median", "value", "unit",
                                                   "accepted_tokens_per_s", "mean_accept_len",
                                                   "hbm_frac", "tflops", "kernels_us_first_layer")}
        out["also"][c5.name]["layers"] = c5.n_layers
    print(json.dumps(out))


def stack_bench(torch, sm, synth, cfg, args):
    """The multi-layer configuration: per layer RMSNorm + MoE verify layer (+ residual), then
    spec_accept; reports end-to-end verify-step latency and accepted tokens per second."""
    x0, layers = synth.make_stack(cfg, "cuda", seed=args.seed)
    draft, target = synth.make_tokens(cfg, seed=args.seed)
    draft_d, target_d = draft.cuda(), target.cuda()
    alen = torch.empty(cfg.B, dtype=torch.int32, device="cuda")
    toks = torch.empty(cfg.B, cfg.gamma + 1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    stack = sm.MoEVerifyStack(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype,
                              renorm=cfg.renorm)

    def step(marks=None, ends=None):
        if ends is not None:
            ends[0].record(stream)
        stack.forward(x0, layers, stream=stream, marks=marks)
        sm.spec_accept(draft_d, target_d, alen, toks, stream)
        if ends is not None:
            ends[1].record(stream)

    for _ in range(args.warmup):
        step()
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    ends = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    if getattr(args, "graph", False):
        graphed = sm.GraphedStep(lambda st: (stack.forward(x0, layers, stream=st),
                                             sm.spec_accept(draft_d, target_d, alen, toks, st)))
        graphed.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graphed.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        for i in range(args.steps):
            step(marks[i], ends[i])
        torch.cuda.synchronize()
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(marks[i], ends[i])
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
    med = statistics.median(a.elapsed_time(b) for a, b in ends)
    names = ("route", "permute", "up", "down", "combine")
    k_us = {n: round(statistics.median(m[j].elapsed_time(m[j + 1]) for m in marks) * 1e3, 2)
            for j, n in enumerate(names)}
    es = 2 if cfg.dtype == "bf16" else 4
    weight_bytes = cfg.n_layers * 3.0 * cfg.E * cfg.d_model * cfg.d_ff * es
    return {
        "metric": "verify_step_accepted_tokens_per_s", "value": float(alen.sum().item()) / (ms * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "ms_per_step_median": med, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "gamma": cfg.gamma, "tokens": cfg.T,
                   "d_model": cfg.d_model, "d_ff": cfg.d_ff, "experts": cfg.E, "top_k": cfg.k,
                   "layers": cfg.n_layers},
        "launch": "hip-graph" if getattr(args, "graph", False) else "eager",
        "accepted_tokens_per_s": float(alen.sum().item()) / (ms * 1e-3),
        "verified_tokens_per_s": cfg.T / (ms * 1e-3),
        "mean_accept_len": float(alen.float().mean().item()),
        "tflops": cfg.flops() * cfg.n_layers / (ms * 1e-3) / 1e12,
        "hbm_frac": weight_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "roofline": {"bound": "hbm", "achieved": weight_bytes / (ms * 1e-3) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": weight_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "kernel": "whole step (weights of all layers streamed once)", "traffic": None},
        "kernels_us_first_layer": k_us,
    }


if __name__ == "__main__":
    main()
