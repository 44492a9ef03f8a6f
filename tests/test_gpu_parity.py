"""Parity of the HIP library (through its C ABI) against the CPU oracle, element by element,
on seeded inputs.  Needs an MI355X:  python -m pytest tests -m gpu"""
import itertools

import numpy as np
import pytest
import torch

import paper_2604_10152_amd as sm
from oracle import moe_verify_oracle as orc
from workloads import synth
from _util import GATE_W_RTOL, TOL, LazyF64, check_float, dev, f64, row_rel_err

pytestmark = pytest.mark.gpu
I32 = torch.int32


def _say(msg):
    print(f"[case] {msg}", flush=True)


# ------------------------------------------------------------------ a5 acceptance
def _gpu_accept(draft, target):
    B, gamma = draft.shape
    alen = torch.full((B,), -7, dtype=I32, device="cuda")
    out = torch.full((B, gamma + 1), -7, dtype=I32, device="cuda")
    sm.spec_accept(dev(draft), dev(target), alen, out)
    torch.cuda.synchronize()
    return alen.cpu().numpy(), out.cpu().numpy()


def test_accept_paper_example_and_exhaustive():
    _say("spec_accept fig4 + exhaustive")
    d = torch.tensor([[10, 11, 12, 13, 14]], dtype=I32)
    t = torch.tensor([[10, 11, 12, 20, 21, 22]], dtype=I32)
    alen, out = _gpu_accept(d, t)
    assert alen.tolist() == [4] and out[0].tolist() == [10, 11, 12, 20, -1, -1]
    for gamma in (1, 3, 7, 10):
        pats = list(itertools.product((0, 1), repeat=gamma))
        draft = torch.arange(len(pats) * gamma, dtype=I32).reshape(len(pats), gamma)
        target = torch.cat([draft + 1 - torch.tensor(pats, dtype=I32),
                            torch.full((len(pats), 1), 777, dtype=I32)], dim=1)
        a, o = _gpu_accept(draft, target)
        ea, eo = orc.accept(draft.numpy(), target.numpy())
        assert (a == ea).all() and (o == eo).all()
        assert a.min() >= 1 and a.max() <= gamma + 1


@pytest.mark.parametrize("cfg_id", [1, 2, 4, 5])
def test_accept_configs(cfg_id):
    cfg = synth.CONFIGS[cfg_id]
    _say(f"spec_accept cfg{cfg_id}")
    draft, target = synth.make_tokens(cfg, seed=cfg_id)
    a, o = _gpu_accept(draft, target)
    ea, eo = orc.accept(draft.numpy(), target.numpy())
    assert (a == ea).all() and (o == eo).all()
    fd, ft = synth.forced_accept_cases(cfg.gamma, cfg.vocab)
    a, o = _gpu_accept(fd, ft)
    assert a.tolist() == list(range(1, cfg.gamma + 2))
    assert (o == orc.accept(fd.numpy(), ft.numpy())[1]).all()


def test_accept_degenerate():
    _say("spec_accept gamma=0, B=0")
    d = torch.zeros((5, 0), dtype=I32)
    t = torch.arange(5, dtype=I32).reshape(5, 1)
    a, o = _gpu_accept(d, t)
    assert a.tolist() == [1] * 5 and o[:, 0].tolist() == [0, 1, 2, 3, 4]
    a, o = _gpu_accept(torch.zeros((0, 3), dtype=I32), torch.zeros((0, 4), dtype=I32))
    assert a.shape == (0,)


# ------------------------------------------------------------------ a1 router
def _gpu_route(x, wr, bias, k, renorm):
    T = x.shape[0]
    idx = torch.full((T, k), -1, dtype=I32, device="cuda")
    w = torch.full((T, k), -1.0, dtype=torch.float32, device="cuda")
    sm.moe_route_topk(dev(x), dev(wr), dev(bias), k, renorm, idx, w)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), w.cpu().numpy()


def _check_route(x, wr, bias, k, renorm):
    idx, w = _gpu_route(x, wr, bias, k, renorm)
    eidx, ew, _ = orc.route_topk(f64(x), f64(wr), k, None if bias is None else f64(bias), renorm)
    assert (idx == eidx).all(), f"{(idx != eidx).sum()} routing indices differ"
    assert np.allclose(w, ew, rtol=GATE_W_RTOL, atol=1e-30)
    if renorm:
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-6)


@pytest.mark.parametrize("dtype,T,d,E,k,renorm,bias", [
    (torch.float32, 16, 256, 8, 2, True, False),
    (torch.float32, 37, 33, 5, 3, False, True),        # d not a multiple of the vector width
    (torch.float32, 9, 8, 1, 1, True, False),
    (torch.bfloat16, 320, 2048, 64, 6, True, True),
    (torch.bfloat16, 130, 192, 130, 7, True, True),    # more experts than lanes
    (torch.bfloat16, 50, 72, 16, 16, False, False),    # k = E
    (torch.bfloat16, 2048, 4096, 8, 2, True, False),
    (torch.bfloat16, 3, 64, 1024, 64, True, True),     # the largest E and k the ABI admits
    (torch.bfloat16, 1500, 128, 20, 2, True, True),    # 4 tokens per workgroup, two expert passes
    (torch.float32, 1100, 40, 9, 2, True, False),      # 4 tokens per workgroup, fp32, odd E
    (torch.bfloat16, 40, 256, 24, 4, True, False),     # 32 experts per pass
    (torch.bfloat16, 2048, 5120, 16, 1, True, True),   # top-1, 16 experts
])
def test_route_cases(dtype, T, d, E, k, renorm, bias):
    _say(f"route {dtype} T={T} d={d} E={E} k={k}")
    g = torch.Generator().manual_seed(T * 31 + E)
    x = (torch.randn(T, d, generator=g) / d ** 0.5).to(dtype)
    wr = torch.randn(E, d, generator=g).to(dtype)
    b = torch.randn(E, generator=g) if bias else None
    _check_route(x, wr, b, k, renorm)


def test_route_ties_go_to_lower_expert_id():
    _say("route ties")
    g = torch.Generator().manual_seed(5)
    x = torch.randn(64, 512, generator=g).to(torch.bfloat16)
    wr = torch.randn(12, 512, generator=g).to(torch.bfloat16)
    wr[7] = wr[2]; wr[11] = wr[2]; wr[5] = wr[0]
    idx, _ = _gpu_route(x, wr, None, 12, True)
    eidx, _, logits = orc.route_topk(f64(x), f64(wr), 12)
    assert (logits[:, 7] == logits[:, 2]).all()
    assert (idx == eidx).all()
    # duplicated rows that meet in different lanes / different passes of the reduction, in the
    # 4-tokens-per-workgroup variant (T >= 1024) and with more experts than one pass holds
    for T2, E2, dup in ((1100, 12, [(7, 2), (11, 2), (5, 0)]), (1100, 40, [(33, 1), (17, 1), (39, 20)]),
                        (70, 100, [(99, 3), (64, 63), (65, 0)])):
        x2 = torch.randn(T2, 256, generator=g).to(torch.bfloat16)
        wr2 = torch.randn(E2, 256, generator=g).to(torch.bfloat16)
        for a, b in dup:
            wr2[a] = wr2[b]
        k2 = min(E2, 12)
        idx2, _ = _gpu_route(x2, wr2, None, k2, True)
        eidx2, _, lg2 = orc.route_topk(f64(x2), f64(wr2), k2)
        assert all((lg2[:, a] == lg2[:, b]).all() for a, b in dup)
        assert (idx2 == eidx2).all(), (T2, E2)
    x0 = torch.zeros(4, 512, dtype=torch.bfloat16)       # all logits equal
    idx0, w0 = _gpu_route(x0, wr, None, 3, True)
    assert (idx0 == np.array([0, 1, 2])).all() and np.allclose(w0, 1 / 3, rtol=1e-6)


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4])
def test_route_configs(cfg_id):
    cfg = synth.CONFIGS[cfg_id]
    _say(f"route cfg{cfg_id}")
    g = torch.Generator().manual_seed(cfg_id)
    x = (torch.randn(cfg.T, cfg.d_model, generator=g) * cfg.x_std).to(cfg.torch_dtype)
    wr = (torch.randn(cfg.E, cfg.d_model, generator=g) * cfg.router_std).to(cfg.torch_dtype)
    bias = None
    if cfg.zipf > 0:
        bias = -cfg.zipf * torch.log(torch.randperm(cfg.E, generator=g).float() + 1)
    _check_route(x, wr, bias, cfg.k, cfg.renorm)


# ------------------------------------------------------------------ a2 permutation
def _gpu_permute(x, idx, E, want_rows=True):
    T, k = idx.shape
    P = T * k
    off = torch.full((E + 1,), -3, dtype=I32, device="cuda")
    rs = torch.full((P,), -3, dtype=I32, device="cuda")
    ro = torch.full((P,), -3, dtype=I32, device="cuda")
    xp = torch.zeros((P, x.shape[1]), dtype=x.dtype, device="cuda") if want_rows else None
    sm.moe_permute(dev(x), dev(idx), E, xp, off, rs, ro)
    torch.cuda.synchronize()
    return off.cpu().numpy(), rs.cpu().numpy(), ro.cpu().numpy(), None if xp is None else xp.cpu()


@pytest.mark.parametrize("dtype,T,d,E,k", [
    (torch.float32, 16, 256, 8, 2),
    (torch.float32, 37, 33, 11, 3),          # ragged everything, 4-byte chunks
    (torch.bfloat16, 37, 17, 11, 3),         # 2-byte chunks
    (torch.bfloat16, 320, 2048, 64, 6),
    (torch.bfloat16, 2048, 4096, 8, 2),
    (torch.bfloat16, 5000, 64, 256, 8),      # many pairs, many experts
    (torch.bfloat16, 1, 64, 1024, 1),
])
def test_permute_cases(dtype, T, d, E, k):
    _say(f"permute {dtype} T={T} d={d} E={E} k={k}")
    rng = np.random.default_rng(T + E)
    # skewed expert popularity with some experts never used
    pop = rng.random(E) ** 3
    pop[rng.random(E) < 0.2] = 0
    pop[0] = max(pop[0], 1e-3)
    if (pop > 0).sum() < k:
        pop[:] = 1.0
    idx = np.stack([rng.choice(E, size=k, replace=False, p=pop / pop.sum()) for _ in range(T)])
    idx_t = torch.from_numpy(idx.astype(np.int32))
    x = torch.randn(T, d, generator=torch.Generator().manual_seed(1)).to(dtype)
    off, rs, ro, xp = _gpu_permute(x, idx_t, E)
    counts, eoff, ers, ero = orc.permute(idx, E)
    assert (off == eoff).all() and (rs == ers).all() and (ro == ero).all()
    assert torch.equal(xp, x[torch.from_numpy(ers.astype(np.int64)) // k])
    assert (np.bincount(rs // k, minlength=T) == k).all()


def test_permute_degenerate():
    _say("permute T=0 and indices-only")
    x = torch.zeros((0, 64), dtype=torch.bfloat16)
    off, rs, ro, _ = _gpu_permute(x, torch.zeros((0, 2), dtype=I32), 8)
    assert (off == 0).all()
    idx = torch.tensor([[1, 0], [1, 2]], dtype=I32)
    off, rs, ro, xp = _gpu_permute(torch.ones(2, 64, dtype=torch.bfloat16), idx, 4, want_rows=False)
    assert off.tolist() == [0, 1, 3, 4, 4] and rs.tolist() == [1, 0, 2, 3] and xp is None


def test_hot_experts_match_oracle():
    """Sec. 3.2 replacement policy input: the N most activated experts, ties to the lower id."""
    _say("hot experts")
    cases = [np.array([3, 9, 9, 1, 9, 0, 9, 2]), np.array([5] * 130), np.arange(70)[::-1] % 7,
             np.array([0, 0, 0, 4])]
    rng = np.random.default_rng(3)
    cases.append(rng.integers(0, 50, size=1024))
    for counts in cases:
        E = len(counts)
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)).cuda()
        for n in sorted({1, min(4, E), E}):
            ids = torch.full((n,), -1, dtype=I32, device="cuda")
            cnt = torch.full((n,), -1, dtype=I32, device="cuda")
            sm.moe_hot_experts(off, ids, cnt)
            torch.cuda.synchronize()
            want = orc.hot_experts(counts, n)
            assert (ids.cpu().numpy() == want).all()
            assert (cnt.cpu().numpy() == counts[want]).all()


# ------------------------------------------------------------------ a3 experts
def _gpu_grouped(xp, off, wg, wu, wd):
    n, d = xp.shape
    E, f, _ = wg.shape
    y = torch.full((n, d), float("nan"), dtype=xp.dtype, device="cuda")
    ws = torch.empty((sm.moe_grouped_swiglu_workspace_bytes(n, d, f, E, xp.dtype),),
                     dtype=torch.uint8, device="cuda")
    sm.moe_grouped_swiglu(dev(xp), dev(off), dev(wg), dev(wu), dev(wd), y, ws)
    torch.cuda.synchronize()
    return y.cpu()


def _grouped_case(dtype, d, f, rows, seed):
    E = len(rows)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    n = int(off[-1])
    g = torch.Generator().manual_seed(seed)
    xp = (torch.randn(n, d, generator=g) / d ** 0.5).to(dtype)
    wg = (torch.randn(E, f, d, generator=g) * 0.5).to(dtype)
    wu = (torch.randn(E, f, d, generator=g) * 0.5).to(dtype)
    wd = (torch.randn(E, d, f, generator=g) * (0.5 / f ** 0.5)).to(dtype)
    y = _gpu_grouped(xp, torch.from_numpy(off), wg, wu, wd)
    ey = orc.grouped_swiglu(f64(xp), off, LazyF64(wg), LazyF64(wu), LazyF64(wd))
    assert torch.isfinite(y.float()).all()
    check_float(f64(y), ey, dtype, f"rows={rows}")


@pytest.mark.parametrize("d,f,rows", [
    (256, 512, [5, 0, 7, 3, 2, 9, 1, 5]),            # cfg-1 shape
    (100, 72, [3, 70, 0, 129]),                      # nothing divides the 64x64x16 tile
    (64, 64, [1]),
])
def test_grouped_fp32(d, f, rows):
    _say(f"grouped f32 d={d} f={f} rows={rows}")
    _grouped_case(torch.float32, d, f, rows, seed=d + f)


@pytest.mark.parametrize("d,f,rows", [
    (256, 384, [300, 0, 37, 1, 513, 256, 330]),      # large-batch tiles: full, ragged, empty
    (512, 1408, [700, 650]),
    (4096, 256, [100, 0, 60, 129, 1, 170]),          # mid tier (128-row tiles) in the gate/up GEMM
    (256, 4096, [100, 0, 60, 129, 1, 170]),          # mid tier in the down GEMM
    (256, 384, [3, 0, 70, 1, 129, 64, 0, 0]),        # few rows per expert: narrow tiles
    (2048, 1408, [0, 40, 1, 0, 310, 7, 0, 22]),      # cfg-3 shape, skewed
    (64, 64, [1]),
])
def test_grouped_bf16(d, f, rows):
    _say(f"grouped bf16 d={d} f={f} rows={rows}")
    _grouped_case(torch.bfloat16, d, f, rows, seed=d + f)


def test_expert_up_alone_matches_swiglu_definition():
    """h = silu(x Wg^T) * (x Wu^T) checked on its own (the gate/up GEMM with its epilogue)."""
    _say("expert up only")
    rows = [200, 0, 61, 300, 420]          # 196 rows per expert on average: large-batch kernel
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    g = torch.Generator().manual_seed(77)
    d, f, E = 256, 384, len(rows)
    xp = (torch.randn(off[-1], d, generator=g) / 16).to(torch.bfloat16)
    wg = torch.randn(E, f, d, generator=g).to(torch.bfloat16)
    wu = torch.randn(E, f, d, generator=g).to(torch.bfloat16)
    h = torch.full((int(off[-1]), f), float("nan"), dtype=torch.bfloat16, device="cuda")
    sm.moe_expert_up_swiglu(dev(xp), dev(torch.from_numpy(off)), dev(wg), dev(wu), h)
    torch.cuda.synchronize()
    x64 = f64(xp)
    want = np.zeros((off[-1], f))
    for e in range(E):
        lo, hi = off[e], off[e + 1]
        want[lo:hi] = orc.silu(x64[lo:hi] @ f64(wg[e]).T) * (x64[lo:hi] @ f64(wu[e]).T)
    check_float(f64(h), want, torch.bfloat16, "up+SwiGLU alone")


# ------------------------------------------------------------------ a4 combine, helpers
@pytest.mark.parametrize("dtype,T,d,k,res", [
    (torch.float32, 16, 256, 2, False), (torch.float32, 7, 33, 3, True),
    (torch.bfloat16, 320, 2048, 6, False), (torch.bfloat16, 33, 4096, 2, True),
    (torch.bfloat16, 5, 24, 4, False),
])
def test_combine(dtype, T, d, k, res):
    _say(f"combine {dtype} T={T} d={d} k={k} residual={res}")
    g = torch.Generator().manual_seed(T + d)
    y = torch.randn(T * k, d, generator=g).to(dtype)
    w = torch.rand(T, k, generator=g)
    w = (w / w.sum(dim=1, keepdim=True)).float()
    ro = torch.randperm(T * k, generator=g).to(I32)
    r = torch.randn(T, d, generator=g).to(dtype) if res else None
    out = torch.empty(T, d, dtype=dtype, device="cuda")
    sm.moe_combine(dev(y), dev(ro), dev(w), dev(r), out)
    torch.cuda.synchronize()
    want = orc.combine(f64(y), ro.numpy(), f64(w), T, k) + (f64(r) if res else 0.0)
    check_float(f64(out), want, dtype, "combine")


@pytest.mark.parametrize("dtype,T,d", [(torch.float32, 5, 100), (torch.bfloat16, 160, 4096)])
def test_rmsnorm(dtype, T, d):
    _say(f"rmsnorm {dtype} T={T} d={d}")
    g = torch.Generator().manual_seed(d)
    x = torch.randn(T, d, generator=g).to(dtype)
    gain = (1 + 0.1 * torch.randn(d, generator=g)).to(dtype)
    out = torch.empty(T, d, dtype=dtype, device="cuda")
    sm.moe_rmsnorm(dev(x), dev(gain), 1e-5, out)
    torch.cuda.synchronize()
    assert row_rel_err(f64(out), orc.rmsnorm(f64(x), f64(gain), 1e-5)) <= TOL[dtype]


# ------------------------------------------------------------------ whole layer
def _run_layer(cfg, L, packed=False):
    """packed: hand the layer tile-packed copies of the expert weights as well (what the
    benchmark does); the layer then runs the projections its plan assigns to them."""
    layer = sm.MoEVerifyLayer(L["x"].shape[0], cfg.d_model, cfg.d_ff, cfg.E, cfg.k,
                              cfg.torch_dtype, renorm=cfg.renorm)
    pk = sm.MoEVerifyLayer.pack_weights(L["w_gate"], L["w_up"], L["w_down"]) if packed else None
    out = layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                        packed=pk)
    torch.cuda.synchronize()
    return layer, out


def _check_routing_and_permutation(cfg, L, layer):
    x64 = f64(L["x"])
    bias = None if L["bias"] is None else f64(L["bias"])
    eidx, ew, _ = orc.route_topk(x64, f64(L["w_router"]), cfg.k, bias, cfg.renorm)
    assert (layer.topk_idx.cpu().numpy() == eidx).all()
    assert np.allclose(layer.topk_w.cpu().numpy(), ew, rtol=GATE_W_RTOL, atol=1e-30)
    counts, eoff, ers, ero = orc.permute(eidx, cfg.E)
    assert (layer.expert_offsets.cpu().numpy() == eoff).all()
    assert (layer.row_src.cpu().numpy() == ers).all()
    assert (layer.row_of.cpu().numpy() == ero).all()
    return counts


@pytest.mark.parametrize("cfg_id,packed", [(1, False), (3, False), (3, True)])
def test_layer_full_oracle(cfg_id, packed):
    """Configurations the oracle can evaluate in full in seconds (cfg 3 on row-major operands
    and, as the benchmark runs it, on tile-packed ones)."""
    cfg = synth.CONFIGS[cfg_id]
    _say(f"layer cfg{cfg_id} full packed={packed}")
    L = synth.make_layer(cfg, "cuda", seed=cfg_id)
    layer, out = _run_layer(cfg, L, packed)
    if packed:
        assert layer.x_packed is not None and layer.h_packed is not None
    counts = _check_routing_and_permutation(cfg, L, layer)
    want = orc.moe_layer_stepwise(f64(L["x"]), f64(L["w_router"]), LazyF64(L["w_gate"]),
                                  LazyF64(L["w_up"]), LazyF64(L["w_down"]), cfg.k,
                                  None if L["bias"] is None else f64(L["bias"]), cfg.renorm)
    check_float(f64(out), want, cfg.torch_dtype,
                f"cfg{cfg_id} active={int((counts > 0).sum())}/{cfg.E} "
                f"skew={orc.skewness(counts):.2f} hottest={int(counts.max())}")
    # run twice: deterministic, bit-identical
    out1 = out.clone()
    _, out2 = _run_layer(cfg, L, packed)
    assert torch.equal(out1, out2)


def _seam_rows(offsets, bm_max=320, gran=16):
    """Permuted rows at the places where a tiling mistake would show: first and last row of
    every expert, both sides of each boundary of the even split into m-tiles of at most
    bm_max rows (heights rounded up to the 16-row matrix-instruction granule), and both ends
    of the last 16-row granule of every m-tile."""
    rows = set()
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        M = hi - lo
        if M <= 0:
            continue
        rows.update((lo, hi - 1))
        mt0 = -(-M // bm_max)
        rpt = -(-(-(-M // mt0)) // gran) * gran
        for b in range(lo, hi, rpt):
            end = min(b + rpt, hi)
            rows.update((b, end - 1, max(b, end - gran), max(b, (end - 1) // gran * gran)))
            if b > lo:
                rows.add(b - 1)
    return sorted(rows)


@pytest.mark.parametrize("cfg_id,n_random,packed", [(2, 24, False), (4, 64, True), (6, 64, True),
                                                    (6, 16, False)])
def test_layer_sampled_tokens(cfg_id, n_random, packed):
    """Full-size layers (Mixtral shape; Llama-4-Scout shape with top-1 routing, Table I) in the
    launch configuration the benchmark times: routing and permutation checked in full; outputs
    on a token sample (tokens are independent, so the definition applies row by row).  The
    sample holds the tokens behind the seam rows of the expert kernels' tiling (mapped back
    through the oracle's row_src) plus seeded random tokens."""
    cfg = synth.CONFIGS[cfg_id]
    _say(f"layer cfg{cfg_id} sampled packed={packed}")
    L = synth.make_layer(cfg, "cuda", seed=cfg_id)
    layer, out = _run_layer(cfg, L, packed)
    assert (layer.x_packed is not None) == packed
    _check_routing_and_permutation(cfg, L, layer)
    x64 = f64(L["x"])
    bias = None if L["bias"] is None else f64(L["bias"])
    eidx, _, _ = orc.route_topk(x64, f64(L["w_router"]), cfg.k, bias, cfg.renorm)
    _, eoff, ers, _ = orc.permute(eidx, cfg.E)
    # tiles of at most 320 rows (from 192 rows per expert on average) or 192 rows (below)
    seam_tokens = {int(ers[r]) // cfg.k for bm in (320, 192) for r in _seam_rows(eoff, bm)}
    rng = np.random.default_rng(cfg_id)
    sample = np.array(sorted(seam_tokens | set(rng.choice(cfg.T, size=n_random, replace=False).tolist())))
    print(f"   cfg{cfg_id}: {len(seam_tokens)} seam tokens, {len(sample)} tokens in all", flush=True)
    sel = torch.from_numpy(sample).cuda()
    # grouped by expert so that every expert's weights are widened to fp64 once
    want = orc.moe_layer_stepwise(x64[sample], f64(L["w_router"]), LazyF64(L["w_gate"]),
                                  LazyF64(L["w_up"]), LazyF64(L["w_down"]), cfg.k, bias, cfg.renorm)
    check_float(f64(out[sel]), want, cfg.torch_dtype, f"cfg{cfg_id} sampled rows")
    assert torch.isfinite(out.float()).all()


@pytest.mark.parametrize("name,cfg", [
    ("cfg1-f32", synth.CONFIGS[1]),
    ("bf16-few-rows-short-k", synth.MoEConfig("g1", "bf16", 256, 384, 8, 2, 10, 3, 1 / 16, 0.05, 1.0)),
    ("bf16-few-rows-long-k", synth.MoEConfig("g2", "bf16", 4096, 256, 4, 2, 10, 3, 1 / 64, 0.05, 1.0)),
    ("bf16-large-batch", synth.MoEConfig("g3", "bf16", 256, 384, 4, 2, 150, 3, 1 / 16, 0.05, 1.0)),
])
def test_gather_fused_equals_materialised(name, cfg):
    """moe_expert_up_swiglu_gather(x, row_src) must equal moe_permute(x -> x_perm) followed by
    moe_expert_up_swiglu(x_perm) bit for bit (same kernel, only the row addresses differ); the
    materialised path is itself checked against the oracle above."""
    _say(f"gather fused vs materialised {name}")
    L = synth.make_layer(cfg, "cuda", seed=21)
    outs = []
    for fuse in (True, False):
        layer = sm.MoEVerifyLayer(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype,
                                  renorm=cfg.renorm, fuse_gather=fuse)
        assert layer.fuse_gather == fuse
        out = layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"])
        torch.cuda.synchronize()
        outs.append((out.clone(), layer.h.clone()))
    assert torch.equal(outs[0][1], outs[1][1])
    assert torch.equal(outs[0][0], outs[1][0])
    want = orc.moe_layer_brute_force(f64(L["x"]), f64(L["w_router"]), LazyF64(L["w_gate"]),
                                     LazyF64(L["w_up"]), LazyF64(L["w_down"]), cfg.k)
    check_float(f64(outs[0][0]), want, cfg.torch_dtype, name)


def test_identical_experts_invariant_on_gpu():
    """All experts share weights + renormalised gates => out = FFN(x) whatever the routing."""
    _say("layer identical experts")
    cfg = synth.MoEConfig("ident", "bf16", 256, 384, 6, 3, 50, 3, 1 / 16, 0.05, 1.0)
    L = synth.make_layer(cfg, "cuda", seed=9)
    for n in ("w_gate", "w_up", "w_down"):
        L[n] = L[n][:1].expand(cfg.E, -1, -1).contiguous()
    layer, out = _run_layer(cfg, L)
    want = orc.expert_ffn(f64(L["x"]), f64(L["w_gate"][0]), f64(L["w_up"][0]), f64(L["w_down"][0]))
    check_float(f64(out), want, torch.bfloat16, "identical experts")


# ------------------------------------------------------------------ multi-layer stack (cfg 5)
def _check_stack(cfg, n_layers, n_sample, seed):
    """Every layer of the stack is checked on its own: the oracle gets the GPU's input h_l of
    that layer (exact bf16 values), so routing is compared bit-exactly layer by layer and the
    outputs h_{l+1} to the single-layer bar.  (Comparing only the end of a 32-layer chain would
    mix in discrete routing flips of near-tie tokens caused by earlier bf16 roundings.)"""
    x, layers = synth.make_stack(cfg, "cuda", seed=seed, n_layers=n_layers)
    stack = sm.MoEVerifyStack(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype,
                              renorm=cfg.renorm)
    out, hidden = stack.forward(x, layers, keep_hidden=True)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    rng = np.random.default_rng(seed)
    sample = np.sort(rng.choice(cfg.T, size=n_sample, replace=False))
    sel = torch.from_numpy(sample).cuda()
    worst = 0.0
    for l, L in enumerate(layers):
        h_in = f64(hidden[l][sel])
        lay = dict(gain=f64(L["gain"]), w_router=f64(L["w_router"]), bias=None,
                   w_gate=LazyF64(L["w_gate"]), w_up=LazyF64(L["w_up"]), w_down=LazyF64(L["w_down"]))
        want = orc.decoder_stack(h_in, [lay], cfg.k, cfg.renorm)
        got = f64(hidden[l + 1][sel])
        # the residual dominates h; judge the layer on what it ADDED, against that increment
        inc_err = row_rel_err(got - h_in, want - h_in)
        worst = max(worst, inc_err)
        print(f"   layer {l}: increment err {inc_err:.3e}", flush=True)
        # rounding h_{l+1} to bf16 costs up to 2^-9 of |h|, which may exceed 1e-2 of the increment
        ulp_floor = float((np.abs(want).max(axis=1) * 2.0 ** -8 / np.abs(want - h_in).max(axis=1)).max())
        assert inc_err <= TOL[cfg.torch_dtype] + ulp_floor, (l, inc_err, ulp_floor)
        assert row_rel_err(got, want) <= TOL[cfg.torch_dtype]
    return worst


def test_stack_three_layers_full_width():
    cfg = synth.CONFIGS[5]
    _say("stack cfg5 shape, 3 layers, 8 sampled tokens")
    _check_stack(cfg, n_layers=3, n_sample=8, seed=5)


def test_stack_small_fp32_all_tokens():
    _say("stack fp32 small, 4 layers")
    cfg = synth.MoEConfig("stack-f32", "f32", 96, 160, 6, 2, 5, 3, 1.0, 0.05, 0.3, n_layers=4)
    _check_stack(cfg, n_layers=4, n_sample=cfg.T, seed=6)


@pytest.mark.timeout(400)
def test_stack_full_32_layers_two_tokens():
    """Configuration 5 at its real depth: 32 resident layers (90 GB of weights), every layer
    checked on two sampled tokens."""
    cfg = synth.CONFIGS[5]
    _say("stack cfg5 full: 32 layers, 2 sampled tokens")
    _check_stack(cfg, n_layers=32, n_sample=2, seed=5)


def test_graph_replay_equals_eager():
    """The multi-layer step captured in a HIP graph: every replay (with eager work and
    synchronisations in between, and with the input refreshed in place) must reproduce the
    eager result bit for bit."""
    _say("HIP graph replay of a 3-layer stack + spec_accept")
    cfg = synth.MoEConfig("graph", "bf16", 256, 384, 8, 2, 12, 3, 1.0, 0.05, 0.5, n_layers=3,
                          match_prob=0.6)
    x, layers = synth.make_stack(cfg, "cuda", seed=9)
    draft, target = synth.make_tokens(cfg, seed=9)
    draft, target = draft.cuda(), target.cuda()
    stack = sm.MoEVerifyStack(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype)
    alen = torch.empty((cfg.B,), dtype=I32, device="cuda")
    toks = torch.empty((cfg.B, cfg.gamma + 1), dtype=I32, device="cuda")
    result = {}

    def step(stream):
        result["out"] = stack.forward(x, layers, stream=stream)
        sm.spec_accept(draft, target, alen, toks, stream)

    step(None)
    torch.cuda.synchronize()
    eager0 = result["out"].clone()
    alen0 = alen.clone()
    g = sm.GraphedStep(step)
    out_buf = result["out"]                       # the buffer the captured step writes
    x_alt = (x.float() * 0.5 + 0.1).to(x.dtype)
    x_orig = x.clone()
    for rep in range(4):
        use_alt = rep % 2 == 1
        x.copy_(x_alt if use_alt else x_orig)
        out_buf.fill_(float("nan"))
        alen.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out_buf.clone()
        # eager reference for the same input, computed after the replay
        step(None)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), result["out"].view(torch.int16)), rep
        assert torch.equal(alen, alen0)
        if not use_alt:
            assert torch.equal(got.view(torch.int16), eager0.view(torch.int16))


def test_zero_sizes_and_single_hot_expert():
    """Degenerate shapes through the whole ABI: no tokens at all (every call is a no-op that leaves
    its outputs alone, moe_permute still writes offsets), and a batch in which ONE expert takes
    every row (all other experts empty) in both dtypes."""
    _say("zero tokens / one expert takes everything")
    E, d, f, k = 4, 64, 128, 2
    for dtype in (torch.float32, torch.bfloat16):
        g = torch.Generator().manual_seed(3)
        wr = torch.randn(E, d, generator=g).to(dtype).cuda()
        wg = (torch.randn(E, f, d, generator=g) * 0.1).to(dtype).cuda()
        wu = (torch.randn(E, f, d, generator=g) * 0.1).to(dtype).cuda()
        wd = (torch.randn(E, d, f, generator=g) * 0.1).to(dtype).cuda()
        x0 = torch.zeros((0, d), dtype=dtype, device="cuda")
        idx0 = torch.zeros((0, k), dtype=I32, device="cuda")
        w0 = torch.zeros((0, k), dtype=torch.float32, device="cuda")
        sm.moe_route_topk(x0, wr, None, k, True, idx0, w0)
        off = torch.full((E + 1,), 9, dtype=I32, device="cuda")
        sm.moe_permute(x0, idx0, E, x0.new_zeros((0, d)), off, idx0.new_zeros((0,)), idx0.new_zeros((0,)))
        y0 = torch.zeros((0, d), dtype=dtype, device="cuda")
        ws = torch.empty((sm.moe_grouped_swiglu_workspace_bytes(0, d, f, E, dtype),), dtype=torch.uint8,
                         device="cuda")
        sm.moe_grouped_swiglu(x0, off, wg, wu, wd, y0, ws)
        out0 = torch.full((0, d), 1.0, dtype=dtype, device="cuda")
        sm.moe_combine(y0, idx0.new_zeros((0,)), w0, None, out0)
        torch.cuda.synchronize()
        assert off.tolist() == [0] * (E + 1)
        # one expert (id 2) receives every row: bias forces it into slot 0 for every token, the
        # second slot is spread by the router
        T = 150
        x = (torch.randn(T, d, generator=g) / 8).to(dtype).cuda()
        bias = torch.tensor([0.0, 0.0, 50.0, 0.0], device="cuda")
        layer = sm.MoEVerifyLayer(T, d, f, E, 1, dtype)
        out = layer.forward(x, wr, wg, wu, wd, bias)
        torch.cuda.synchronize()
        assert layer.expert_offsets.tolist() == [0, 0, 0, T, T]
        want = orc.moe_layer_brute_force(f64(x), f64(wr), f64(wg), f64(wu), f64(wd), 1, f64(bias), True)
        assert (layer.topk_idx.cpu().numpy() == 2).all()
        check_float(f64(out), want, dtype, "one hot expert")


# ------------------------------------------------------------------ tile-packed operands
def _tile_packed(w):
    """The packed layout written out from its definition (test side): 1 KB blocks of 16 rows x 32
    columns, block (rb, kb) at (rb * K/32 + kb), chunk c of row r at piece 4r + (c ^ ((r/2)%4))."""
    a = w.view(torch.int16).cpu().numpy()
    E, R, K = a.shape
    out = np.empty_like(a).reshape(E, R // 16, K // 32, 64, 8)
    blocks = a.reshape(E, R // 16, 16, K // 32, 4, 8)            # [E, rb, r, kb, c, 8]
    for r in range(16):
        for c in range(4):
            out[:, :, :, 4 * r + (c ^ ((r // 2) % 4)), :] = blocks[:, :, r, :, c, :]
    return out.reshape(E, R, K)


@pytest.mark.parametrize("E,R,K", [(3, 64, 96), (2, 384, 256), (1, 16, 32)])
def test_pack_weights_layout(E, R, K):
    _say(f"pack weights {E}x{R}x{K}")
    g = torch.Generator().manual_seed(R + K)
    w = torch.randn(E, R, K, generator=g).to(torch.bfloat16).cuda()
    wp = torch.full_like(w, float("nan"))
    sm.moe_pack_weights(w, wp)
    torch.cuda.synchronize()
    assert (wp.view(torch.int16).cpu().numpy() == _tile_packed(w)).all()


@pytest.mark.parametrize("d,f,rows", [
    (256, 384, [300, 0, 37, 1, 513, 256, 330]),      # full, ragged, empty experts; padded blocks
    (512, 1408, [700, 650]),
    (256, 384, [3, 0, 70, 1, 129, 64, 0, 0]),        # few rows: still correct on the packed path
    (64, 64, [1]),
    # more experts than lanes: the block numbering carries over the 64-expert sweeps of the scans
    (128, 128, [(7 * e) % 23 if e % 3 else 0 for e in range(130)]),
    (128, 64, [0] * 70 + [200, 17] + [0] * 60 + [33]),
    # few rows per expert, longer contractions: ragged and empty experts on the 192-row tiles
    (256, 512, [3, 0, 70, 1, 129, 64, 0, 0]),
    (128, 256, [5, 17, 64, 1, 0, 33, 65, 16]),
    (512, 1024, [40, 1]),
])
def test_packed_expert_gemms(d, f, rows):
    """moe_expert_up_swiglu_gather_packed + moe_expert_down_packed against the oracle, and - where
    the row-major entry points pick the same large-batch kernel - bit for bit against them."""
    _say(f"packed expert GEMMs d={d} f={f} rows={rows}")
    E = len(rows)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    n = int(off[-1])
    g = torch.Generator().manual_seed(d + f + n)
    xp = (torch.randn(n, d, generator=g) / d ** 0.5).to(torch.bfloat16)
    wg = (torch.randn(E, f, d, generator=g) * 0.5).to(torch.bfloat16)
    wu = (torch.randn(E, f, d, generator=g) * 0.5).to(torch.bfloat16)
    wd = (torch.randn(E, d, f, generator=g) * (0.5 / f ** 0.5)).to(torch.bfloat16)
    doff = dev(torch.from_numpy(off))
    pk = sm.MoEVerifyLayer.pack_weights(dev(wg), dev(wu), dev(wd))
    hp = torch.full((sm.moe_packed_h_bytes(n, f, E),), 0xff, dtype=torch.uint8, device="cuda")
    y = torch.full((n, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    sm.moe_expert_up_swiglu_gather_packed(dev(xp), None, 1, doff, pk["w_gate"], pk["w_up"], n, hp)
    sm.moe_expert_down_packed(hp, doff, pk["w_down"], y)
    # the same with the activation rows gathered into tile-packed form first: identical bits
    hp2 = torch.full_like(hp, 0xee)
    xws = torch.full((sm.moe_packed_h_bytes(n, d, E),), 0xdd, dtype=torch.uint8, device="cuda")
    y3 = torch.full_like(y, float("nan"))
    sm.moe_expert_up_swiglu_gather_packed(dev(xp), None, 1, doff, pk["w_gate"], pk["w_up"], n, hp2, xws)
    sm.moe_expert_down_packed(hp2, doff, pk["w_down"], y3)
    # ... and as the two calls of their own (permute step writes the packed rows, then the GEMM)
    hp3 = torch.full_like(hp, 0xcc)
    xws3 = torch.full_like(xws, 0xbb)
    sm.moe_permute_rows_packed(dev(xp), None, 1, doff, n, xws3)
    sm.moe_expert_up_swiglu_packed(xws3, doff, pk["w_gate"], pk["w_up"], n, hp3)
    # ... and with h written row-major for the row-major down projection
    h_rm = torch.full((n, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    y4 = torch.full_like(y, float("nan"))
    sm.moe_expert_up_swiglu_packed(xws3, doff, pk["w_gate"], pk["w_up"], n, h_rm, h_row_major=True)
    sm.moe_expert_down(h_rm, doff, dev(wd), y4)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y3.view(torch.int16))
    used = (sum((r + 15) // 16 for r in rows)) * 16 * f * 2          # blocks the batch really uses
    assert torch.equal(hp[:used], hp2[:used])
    assert torch.equal(hp[:used], hp3[:used])
    usedx = used // f * d
    assert torch.equal(xws[:usedx], xws3[:usedx])
    # the packed rows are the tile-packed image of x_perm, padding rows zero
    xpad = torch.zeros(usedx // (2 * d), d, dtype=torch.bfloat16)
    b = 0
    for e, r in enumerate(rows):
        xpad[16 * b:16 * b + r] = xp[off[e]:off[e + 1]]
        b += (r + 15) // 16
    assert (xws3[:usedx].cpu().view(torch.int16).numpy() ==
            _tile_packed(xpad[None]).reshape(-1)).all()
    # row-major h = the packed h, un-tiled (same kernel arithmetic, only the store differs)
    hpad = torch.zeros(used // (2 * f), f, dtype=torch.bfloat16)
    b = 0
    for e, r in enumerate(rows):
        hpad[16 * b:16 * b + r] = h_rm[off[e]:off[e + 1]].cpu()
        b += (r + 15) // 16
    assert (hp3[:used].cpu().view(torch.int16).numpy() == _tile_packed(hpad[None]).reshape(-1)).all()
    ey = orc.grouped_swiglu(f64(xp), off, LazyF64(wg), LazyF64(wu), LazyF64(wd))
    check_float(f64(y), ey, torch.bfloat16, f"packed rows={rows}")
    check_float(f64(y4), ey, torch.bfloat16, f"packed up, row-major down rows={rows}")
    if n >= 192 * E:
        y2 = _gpu_grouped(xp, torch.from_numpy(off), wg, wu, wd)
        assert torch.equal(y.cpu().view(torch.int16), y2.view(torch.int16))


def test_layer_cfg4_packed_path():
    """The benchmark workload on the tile-packed path: same routing, output bit-identical to the
    row-major path (same kernels' arithmetic in the same order)."""
    cfg = synth.CONFIGS[4]
    _say("layer cfg4 packed")
    L = synth.make_layer(cfg, "cuda", seed=4)
    layer, out = _run_layer(cfg, L)
    ref = out.clone()
    pk = sm.MoEVerifyLayer.pack_weights(L["w_gate"], L["w_up"], L["w_down"])
    out2 = layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                         packed=pk)
    torch.cuda.synchronize()
    assert layer.h_packed is not None
    assert torch.equal(ref.view(torch.int16), out2.view(torch.int16))


@pytest.mark.parametrize("name,cfg,plan", [
    ("short-k-all-packed", synth.MoEConfig("p1", "bf16", 256, 384, 8, 2, 10, 3, 1 / 16, 0.05, 1.0),
     (True, True)),
    ("up-packed-down-row-major", synth.MoEConfig("p2", "bf16", 256, 4096, 4, 2, 25, 3, 1 / 16, 0.05, 1.0),
     (True, False)),
    ("long-k-96-rows-all-packed", synth.MoEConfig("p3", "bf16", 256, 4096, 2, 2, 25, 3, 1 / 16, 0.05, 1.0),
     (True, True)),
    ("long-k-few-rows-row-major", synth.MoEConfig("p4", "bf16", 4096, 256, 4, 2, 10, 3, 1 / 64, 0.05, 1.0),
     (False, False)),
])
def test_layer_packed_plans(name, cfg, plan):
    """Every combination the layer's plan can pick (gate/up and down each on tile-packed or on
    row-major operands, h in the layout the down projection reads) against the full oracle."""
    _say(f"layer packed plan {name}")
    assert sm.MoEVerifyLayer.packed_plan(cfg.T * cfg.k, cfg.E, cfg.d_model, cfg.d_ff) == plan
    L = synth.make_layer(cfg, "cuda", seed=31)
    layer, out = _run_layer(cfg, L, packed=True)
    assert (layer.x_packed is not None) == plan[0]
    assert (layer.h_packed is not None) == plan[1]
    _check_routing_and_permutation(cfg, L, layer)
    want = orc.moe_layer_brute_force(f64(L["x"]), f64(L["w_router"]), LazyF64(L["w_gate"]),
                                     LazyF64(L["w_up"]), LazyF64(L["w_down"]), cfg.k)
    check_float(f64(out), want, cfg.torch_dtype, name)
