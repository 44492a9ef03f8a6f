"""Parity of the speculation-phase and verification-rule entry points (affinity table, nearest
draft expert, draft routing, sampling-based acceptance, greedy head, active-expert volume)
against the CPU oracle.  Needs an MI355X:  python -m pytest tests -m gpu"""
import numpy as np
import pytest
import torch

import paper_2604_10152_amd as sm
from oracle import moe_verify_oracle as orc
from workloads import synth
from _util import TOL, LazyF64, dev, f64, row_rel_err

pytestmark = pytest.mark.gpu
I32 = torch.int32
AFFINITY_RTOL = 1e-6     # fp64 sums on both sides, one rounding of the distance to fp32;
                         # the kernel squares 4 or 8 differences in fp32 before widening


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _weights(E, d, f, dtype, seed, planted=True):
    g = torch.Generator(device="cpu").manual_seed(seed)
    mk = lambda *shape: (torch.randn(*shape, generator=g) * 0.02).to(dtype)
    wg, wu, wd = mk(E, f, d), mk(E, f, d), mk(E, d, f)
    if planted and E >= 4:
        # expert 3 is a copy of expert 1; expert 2 is expert 0 plus a small perturbation
        for w in (wg, wu, wd):
            w[3] = w[1]
            w[2] = (w[0].float() + 0.002 * torch.randn(w[0].shape, generator=g)).to(dtype)
    return wg, wu, wd


def _gpu_affinity(wg, wu, wd):
    E = wg.shape[0]
    table = torch.full((E, E), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty((sm.moe_affinity_table_workspace_bytes(E),), dtype=torch.uint8, device="cuda")
    sm.moe_affinity_table(dev(wg), dev(wu), dev(wd), table, ws)
    torch.cuda.synchronize()
    return table.cpu().numpy()


# ------------------------------------------------------------------ n2 affinity table
@pytest.mark.parametrize("E,d,f,dtype", [(8, 256, 512, torch.float32), (12, 128, 192, torch.bfloat16),
                                         (5, 64, 64, torch.bfloat16), (64, 128, 64, torch.bfloat16),
                                         (17, 20, 12, torch.float32)])
def test_affinity_table_matches_oracle(E, d, f, dtype):
    _say(f"affinity table E={E} d={d} f={f} {dtype}")
    wg, wu, wd = _weights(E, d, f, dtype, seed=100 + E)
    got = _gpu_affinity(wg, wu, wd)
    want = orc.affinity_table(f64(wg), f64(wu), f64(wd))
    assert np.all(np.diag(got) == 0) and np.array_equal(got, got.T)
    np.testing.assert_allclose(got, want, rtol=AFFINITY_RTOL, atol=0)
    if E >= 4:
        assert got[1, 3] == 0


def test_affinity_table_cfg3_shape_sampled_pairs():
    """Full fine-grained shape (64 experts x 3 x 2048 x 1408, bf16): the oracle evaluates a seeded
    sample of pairs; symmetry and the zero diagonal are checked on the whole table."""
    cfg = synth.CONFIGS[3]
    _say("affinity table cfg3 full shape")
    L = synth.make_layer(cfg, "cuda", seed=3)
    got = _gpu_affinity(L["w_gate"], L["w_up"], L["w_down"])
    assert np.all(np.diag(got) == 0) and np.array_equal(got, got.T) and np.all(np.isfinite(got))
    rng = np.random.default_rng(5)
    for _ in range(6):
        i, j = rng.choice(cfg.E, size=2, replace=False)
        sq = 0.0
        for W in (L["w_gate"], L["w_up"], L["w_down"]):
            sub = orc.affinity_table([f64(W[i]), f64(W[j])], [np.zeros(1)] * 2, [np.zeros(1)] * 2)
            sq += sub[0, 1] ** 2
        assert got[i, j] == pytest.approx(np.sqrt(sq), rel=AFFINITY_RTOL)
    # i.i.d. N(0, 0.02^2) weights: every distance is close to 0.02 * sqrt(2 * 3*d*f)
    off = got[~np.eye(cfg.E, dtype=bool)]
    assert np.allclose(off, 0.02 * np.sqrt(6.0 * cfg.d_model * cfg.d_ff), rtol=5e-3)


# ------------------------------------------------------------------ n2 nearest draft expert
def _gpu_remap(table, draft_ids):
    E = table.shape[0]
    remap = torch.full((E,), -9, dtype=I32, device="cuda")
    sm.moe_nearest_draft_expert(torch.from_numpy(table.astype(np.float32)).cuda(),
                                torch.tensor(draft_ids, dtype=I32, device="cuda"), remap)
    torch.cuda.synchronize()
    return remap.cpu().numpy()


def test_nearest_draft_expert_matches_oracle():
    _say("nearest draft expert")
    rng = np.random.default_rng(11)
    for E in (4, 8, 64, 130, 1024):
        A = rng.integers(1, 6, size=(E, E)).astype(np.float32)      # few values -> many exact ties
        A = np.triu(A, 1) + np.triu(A, 1).T
        for N in sorted({1, 2, max(1, E // 4), E}):
            draft = rng.permutation(E)[:N].tolist()                  # unsorted
            got = _gpu_remap(A, draft)
            want = orc.nearest_draft_expert(A.astype(np.float64), draft)
            assert np.array_equal(got, want), (E, N)
    # ids outside [0, E) are ignored
    A = np.array([[0, 2, 1], [2, 0, 3], [1, 3, 0]], dtype=np.float32)
    assert _gpu_remap(A, [7, 2, -1]).tolist() == [2, 2, 2]


# ------------------------------------------------------------------ n2 draft routing and layer
def _draft_setup(cfg, seed, n_draft):
    """Verification pass -> hot experts -> remap, all on the GPU; returns the pieces."""
    L = synth.make_layer(cfg, "cuda", seed=seed)
    layer = sm.MoEVerifyLayer(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.torch_dtype,
                              renorm=cfg.renorm)
    layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"])
    hot = torch.empty((n_draft,), dtype=I32, device="cuda")
    sm.moe_hot_experts(layer.expert_offsets, hot)
    table = torch.empty((cfg.E, cfg.E), dtype=torch.float32, device="cuda")
    ws = torch.empty((sm.moe_affinity_table_workspace_bytes(cfg.E),), dtype=torch.uint8, device="cuda")
    sm.moe_affinity_table(L["w_gate"], L["w_up"], L["w_down"], table, ws)
    remap = torch.empty((cfg.E,), dtype=I32, device="cuda")
    sm.moe_nearest_draft_expert(table, hot, remap)
    torch.cuda.synchronize()
    return L, layer, hot, table, remap


@pytest.mark.parametrize("cfg_id,n_draft", [(1, 3), (3, 16), (3, 6), (2, 2)])
def test_draft_routing_matches_oracle(cfg_id, n_draft):
    """The real chain: counts of a verification pass choose the draft experts (HotTemporal), the
    table maps every other expert to one of them, the draft router uses the map.  The oracle
    gets the GPU's fp32 table (the table itself is checked above), so ids must match exactly."""
    cfg = synth.CONFIGS[cfg_id]
    _say(f"draft routing cfg{cfg_id} N={n_draft}")
    L, layer, hot, table, remap = _draft_setup(cfg, seed=cfg_id, n_draft=n_draft)
    counts = np.diff(layer.expert_offsets.cpu().numpy())
    hot_want = orc.hot_experts(counts, n_draft)
    assert np.array_equal(hot.cpu().numpy(), hot_want)
    tab64 = table.cpu().numpy().astype(np.float64)
    assert np.array_equal(remap.cpu().numpy(), orc.nearest_draft_expert(tab64, hot_want))
    idx = torch.full((cfg.T, cfg.k), -1, dtype=I32, device="cuda")
    w = torch.full((cfg.T, cfg.k), -1.0, dtype=torch.float32, device="cuda")
    sm.moe_route_topk_draft(L["x"], L["w_router"], L["bias"], cfg.k, cfg.renorm, remap, idx, w)
    torch.cuda.synchronize()
    bias = None if L["bias"] is None else f64(L["bias"])
    idx_want, w_want = orc.route_topk_draft(f64(L["x"]), f64(L["w_router"]), cfg.k, hot_want,
                                            tab64, bias, cfg.renorm)
    assert np.array_equal(idx.cpu().numpy(), idx_want)
    np.testing.assert_allclose(w.cpu().numpy(), w_want, rtol=2e-6, atol=0)
    assert set(np.unique(idx_want)) <= set(hot_want.tolist())


@pytest.mark.parametrize("cfg_id,n_draft,n_tok", [(1, 3, 16), (3, 16, 24)])
def test_draft_layer_matches_oracle(cfg_id, n_draft, n_tok):
    """Whole MoE block in draft mode (only the N resident experts compute) against the oracle on
    the first n_tok tokens (tokens are independent)."""
    cfg = synth.CONFIGS[cfg_id]
    _say(f"draft layer cfg{cfg_id} N={n_draft}")
    L, layer, hot, table, remap = _draft_setup(cfg, seed=cfg_id, n_draft=n_draft)
    out = layer.forward(L["x"], L["w_router"], L["w_gate"], L["w_up"], L["w_down"], L["bias"],
                        draft_remap=remap)
    torch.cuda.synchronize()
    counts = np.diff(layer.expert_offsets.cpu().numpy())
    assert set(np.nonzero(counts)[0].tolist()) <= set(hot.cpu().numpy().tolist())
    bias = None if L["bias"] is None else f64(L["bias"])
    want, idx_want, _ = orc.moe_layer_draft(
        f64(L["x"][:n_tok]), f64(L["w_router"]), LazyF64(L["w_gate"]), LazyF64(L["w_up"]),
        LazyF64(L["w_down"]), cfg.k, hot.cpu().numpy(), table.cpu().numpy().astype(np.float64),
        bias, cfg.renorm)
    assert np.array_equal(layer.topk_idx[:n_tok].cpu().numpy(), idx_want)
    err = row_rel_err(out[:n_tok].float().cpu().numpy(), want)
    print(f"   draft layer row error {err:.3e}")
    assert err <= TOL[cfg.torch_dtype]


# ------------------------------------------------------------------ n3 sampling-based acceptance
def _gpu_accept_sample(draft, pd, pt, ua, us):
    B, gp1, V = pt.shape
    alen = torch.full((B,), -7, dtype=I32, device="cuda")
    out = torch.full((B, gp1), -7, dtype=I32, device="cuda")
    sm.spec_accept_sample(dev(draft), dev(pd), dev(pt), dev(ua), dev(us), alen, out)
    torch.cuda.synchronize()
    return alen.cpu().numpy(), out.cpu().numpy()


def _draw_is_valid(weights, u, tok):
    """tok is a correct inverse-CDF draw up to the rounding of the running sums."""
    c = np.cumsum(np.asarray(weights, dtype=np.float64))
    thr = np.float64(u) * c[-1]
    below = c[tok - 1] if tok > 0 else 0.0
    return weights[tok] > 0 and below <= thr * (1 + 1e-12) and c[tok] >= thr * (1 - 1e-12)


def _sample_case(B, gamma, V, seed, sharp=1.0, agree=0.6):
    g = torch.Generator(device="cpu").manual_seed(seed)
    pt = torch.softmax(torch.randn(B, gamma + 1, V, generator=g) * sharp, dim=-1)
    pd = torch.softmax(torch.log(pt[:, :gamma]) + 0.7 * torch.randn(B, gamma, V, generator=g), dim=-1)
    draft = torch.multinomial(pd.reshape(-1, V), 1, generator=g).reshape(B, gamma).to(I32) \
        if gamma > 0 else torch.zeros((B, 0), dtype=I32)
    ua = torch.rand(B, gamma, generator=g)
    us = torch.rand(B, generator=g)
    return draft, pd.contiguous(), pt.contiguous(), ua, us


@pytest.mark.parametrize("B,gamma,V,sharp", [(64, 5, 1000, 2.0), (8, 7, 32000, 3.0), (33, 1, 17, 1.0),
                                              (16, 0, 50, 1.0), (4, 64, 300, 2.0), (256, 7, 4096, 4.0)])
def test_accept_sample_matches_oracle(B, gamma, V, sharp):
    _say(f"spec_accept_sample B={B} gamma={gamma} V={V}")
    draft, pd, pt, ua, us = _sample_case(B, gamma, V, seed=B * 131 + gamma, sharp=sharp)
    a, o = _gpu_accept_sample(draft, pd, pt, ua, us)
    ea, eo = orc.accept_sample(draft.numpy(), pd.numpy(), pt.numpy(), ua.numpy(), us.numpy())
    assert np.array_equal(a, ea)                       # the keep tests are exact on both sides
    assert a.min() >= 1 and a.max() <= gamma + 1
    if gamma >= 5 and B >= 64:
        assert len(np.unique(a)) >= 3                  # the case exercises several lengths
    for b in range(B):
        n = ea[b] - 1
        assert np.array_equal(o[b, :n], eo[b, :n]) and np.all(o[b, n + 1:] == -1)
        if o[b, n] != eo[b, n]:                        # only legitimate on a rounding boundary
            wts = np.maximum(pt[b, n].double().numpy() - pd[b, n].double().numpy(), 0) \
                if n < gamma else pt[b, n].double().numpy()
            assert _draw_is_valid(wts, us[b].item(), int(o[b, n])), (b, o[b, n], eo[b, n])


def test_accept_sample_special_cases():
    _say("spec_accept_sample special cases")
    # point masses: the rule is the greedy rule (worked example of Fig. 4 included)
    V, gamma = 40, 5
    rng = np.random.default_rng(9)
    draft = rng.integers(0, V, size=(50, gamma)).astype(np.int32)
    target = rng.integers(0, V, size=(50, gamma + 1)).astype(np.int32)
    keep = rng.random(size=(50, gamma)) < 0.75
    target[:, :gamma] = np.where(keep, draft, target[:, :gamma])
    draft[0] = [10, 11, 12, 13, 14]
    target[0] = [10, 11, 12, 20, 21, 22]
    oh = lambda ids: torch.nn.functional.one_hot(torch.from_numpy(ids).long(), V).float()
    a, o = _gpu_accept_sample(torch.from_numpy(draft), oh(draft), oh(target),
                              torch.rand(50, gamma), torch.rand(50))
    ga, go = orc.accept(draft, target)
    assert np.array_equal(a, ga) and np.array_equal(o, go)
    assert a[0] == 4 and o[0].tolist() == [10, 11, 12, 20, -1, -1]
    # identical distributions: nothing can be rejected
    d2, pd, pt, ua, us = _sample_case(20, 4, 64, seed=77)
    pt[:, :4] = pd
    a, o = _gpu_accept_sample(d2, pd, pt, ua, us)
    assert np.all(a == 5) and np.array_equal(o[:, :4], d2.numpy())
    # a draft id outside the vocabulary is rejected at once
    d3 = d2.clone()
    d3[:, 0] = 64
    a, o = _gpu_accept_sample(d3, pd, pt, ua, us)
    assert np.all(a == 1) and np.all((o[:, 0] >= 0) & (o[:, 0] < 64)) and np.all(o[:, 1:] == -1)


# ------------------------------------------------------------------ n4 greedy head, active volume
@pytest.mark.parametrize("R,V,dtype", [(64, 32000, torch.bfloat16), (7, 1001, torch.bfloat16),
                                       (33, 4096, torch.float32), (5, 13, torch.float32),
                                       (2048, 32000, torch.bfloat16)])
def test_greedy_tokens_match_oracle(R, V, dtype):
    _say(f"spec_greedy_tokens R={R} V={V} {dtype}")
    g = torch.Generator(device="cuda").manual_seed(R + V)
    logits = (torch.randn(R, V, generator=g, device="cuda") * 3).to(dtype)
    if R <= 64:
        logits = torch.round(logits * 2) / 2            # coarse grid: many exact ties at the top
        logits = logits.to(dtype)
    tok = torch.full((R,), -5, dtype=I32, device="cuda")
    sm.spec_greedy_tokens(logits, tok)
    torch.cuda.synchronize()
    rows = range(R) if R <= 64 else range(0, R, 37)
    lf = logits.float().cpu().numpy()
    want = orc.greedy_tokens(lf[list(rows)])
    assert np.array_equal(tok.cpu().numpy()[list(rows)], want)
    # property at any size: the chosen logit is the row maximum and no lower id attains it
    mx = lf.max(axis=1)
    t = tok.cpu().numpy()
    assert np.all(lf[np.arange(R), t] == mx)
    assert np.all(t == (lf == mx[:, None]).argmax(axis=1))


def test_active_expert_bytes_and_greedy_accept_chain():
    _say("active expert bytes + greedy head feeding spec_accept")
    for counts in ([3, 0, 5, 0, 0, 1, 2, 9], [0] * 64, list(range(130))):
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)).cuda()
        out = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        per = 3 * 4096 * 14336 * 2
        sm.moe_active_expert_bytes(off, per, out)
        torch.cuda.synchronize()
        assert int(out.item()) == orc.active_expert_bytes(counts, per)
    # logits -> greedy target tokens -> greedy acceptance, against the oracle's chain
    B, gamma, V = 32, 4, 500
    g = torch.Generator(device="cpu").manual_seed(5)
    logits = torch.randn(B * (gamma + 1), V, generator=g)
    tgt_want = orc.greedy_tokens(logits.numpy()).reshape(B, gamma + 1)
    draft = torch.from_numpy(tgt_want[:, :gamma].copy())
    flip = torch.rand(B, gamma, generator=g) < 0.3
    draft = torch.where(flip, (draft + 1) % V, draft).to(I32)
    tok = torch.empty((B * (gamma + 1),), dtype=I32, device="cuda")
    sm.spec_greedy_tokens(logits.cuda(), tok)
    alen = torch.empty((B,), dtype=I32, device="cuda")
    out = torch.empty((B, gamma + 1), dtype=I32, device="cuda")
    sm.spec_accept(draft.cuda(), tok.view(B, gamma + 1), alen, out)
    torch.cuda.synchronize()
    ea, eo = orc.accept(draft.numpy(), tgt_want)
    assert np.array_equal(alen.cpu().numpy(), ea) and np.array_equal(out.cpu().numpy(), eo)
