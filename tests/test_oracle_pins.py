"""Pins of the CPU oracle to things other than itself: the paper's worked example, closed
forms, library routines, exact rational arithmetic, brute force and invariants.  CPU only."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import moe_verify_oracle as orc
from workloads import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _tiny_layer(seed, T=7, d=6, f=10, E=5):
    r = _rng(seed)
    return dict(x=r.normal(size=(T, d)), wr=r.normal(size=(E, d)),
                wg=r.normal(size=(E, f, d)) * 0.5, wu=r.normal(size=(E, f, d)) * 0.5,
                wd=r.normal(size=(E, d, f)) * 0.5)


# ---------------------------------------------------------------- acceptance (a5)
def _read_golden(name):
    rec = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rec[key] = [int(v) for v in vals]
    return rec


def test_accept_paper_worked_example():
    """Fig. 4: 5 drafts, earliest rejection at the 4th -> 3 accepted, 4 generated."""
    g = _read_golden("fig4_accept.txt")
    gamma = g["gamma"][0]
    draft = np.array([g["draft"]], dtype=np.int32)
    target = np.array([g["target"]], dtype=np.int32)
    assert draft.shape == (1, gamma) and target.shape == (1, gamma + 1)
    alen, out = orc.accept(draft, target)
    assert alen[0] == g["generated"][0]
    assert alen[0] - 1 == g["accepted"][0]
    assert out[0].tolist() == g["out_tokens"]


@pytest.mark.parametrize("gamma", [0, 1, 2, 3, 5, 7])
def test_accept_exhaustive_match_patterns(gamma):
    """All 2^gamma match/mismatch patterns; expectation from the pattern string itself."""
    pats = list(itertools.product("01", repeat=gamma))
    B = len(pats)
    draft = np.arange(B * gamma, dtype=np.int32).reshape(B, gamma) * 3 + 5
    target = np.zeros((B, gamma + 1), dtype=np.int32)
    target[:, gamma] = 99999
    for b, pat in enumerate(pats):
        for i, c in enumerate(pat):
            target[b, i] = draft[b, i] if c == "1" else draft[b, i] + 1
    alen, out = orc.accept(draft, target)
    for b, pat in enumerate(pats):
        s = "".join(pat)
        n = s.find("0") if "0" in s else gamma
        assert alen[b] == n + 1
        assert 1 <= alen[b] <= gamma + 1
        assert out[b, :n + 1].tolist() == target[b, :n + 1].tolist()
        assert (out[b, n + 1:] == -1).all()


@pytest.mark.parametrize("gamma,expect", [(3, 2.533), (4, 2.7731), (7, 3.1412), (10, 3.2674)])
def test_accept_mean_matches_geometric_closed_form(gamma, expect):
    """i.i.d. per-position match probability p: E[accept_len] = (1 - p^(gamma+1)) / (1 - p)."""
    p = 0.7
    closed = (1 - p ** (gamma + 1)) / (1 - p)
    assert abs(closed - expect) < 5e-4
    cfg = synth.MoEConfig("t", "f32", 8, 8, 2, 1, 200000, gamma, 1, 1, 1, match_prob=p)
    draft, target = synth.make_tokens(cfg, seed=3)
    alen, _ = orc.accept(draft.numpy(), target.numpy())
    # var(accept_len) < gamma^2; 5 sigma of the mean over 2e5 samples
    assert abs(alen.mean() - closed) < 5 * gamma / np.sqrt(200000)


def test_accept_forced_cases_and_shape_check():
    draft, target = synth.forced_accept_cases(4)
    alen, out = orc.accept(draft.numpy(), target.numpy())
    assert alen.tolist() == [1, 2, 3, 4, 5]
    with pytest.raises(ValueError):
        orc.accept(np.zeros((2, 3), np.int32), np.zeros((2, 3), np.int32))


# ---------------------------------------------------------------- router (a1)
def test_router_logits_exact_rational():
    """Exact rational arithmetic on a tiny non-square case (pins operand orientation + bias)."""
    r = _rng(1)
    x = r.integers(-8, 9, size=(3, 4)) / 8.0
    wr = r.integers(-8, 9, size=(5, 4)) / 16.0
    bias = r.integers(-8, 9, size=5) / 4.0
    got = orc.router_logits(x, wr, bias)
    for t in range(3):
        for e in range(5):
            want = Fraction(float(bias[e])) + sum(Fraction(float(x[t, j])) * Fraction(float(wr[e, j]))
                                                  for j in range(4))
            assert got[t, e] == float(want)


def test_topk_matches_stable_library_argsort():
    r = _rng(2)
    logits = r.normal(size=(200, 16))
    logits[::3, 5] = logits[::3, 2]          # planted exact ties
    logits[::7, 11] = logits[::7, 0]
    for k in (1, 2, 6, 16):
        idx = orc.topk_of_logits(logits, k)
        ref = np.argsort(-logits, axis=1, kind="stable")[:, :k]
        assert (idx == ref).all()


def test_topk_invariants():
    r = _rng(3)
    logits = r.normal(size=(64, 12))
    k = 4
    idx = orc.topk_of_logits(logits, k)
    for t in range(64):
        sel = idx[t].tolist()
        assert len(set(sel)) == k
        vals = logits[t, sel]
        assert (np.diff(vals) <= 0).all()
        rest = np.delete(logits[t], sel)
        assert rest.max() <= vals[-1]


def test_gate_renorm_equals_softmax_over_selected():
    r = _rng(4)
    logits = r.normal(size=(50, 9)) * 3
    idx = orc.topk_of_logits(logits, 3)
    w = orc.gate_weights(logits, idx, renorm=True)
    sel = np.take_along_axis(logits, idx.astype(np.int64), axis=1)
    assert np.allclose(w, scipy.special.softmax(sel, axis=1), rtol=1e-13, atol=0)
    assert np.allclose(w.sum(axis=1), 1.0, rtol=1e-14)


def test_gate_special_cases():
    r = _rng(5)
    logits = r.normal(size=(20, 6))
    # k = E: the full softmax, ordered by descending probability
    idx = orc.topk_of_logits(logits, 6)
    w = orc.gate_weights(logits, idx, renorm=False)
    full = scipy.special.softmax(logits, axis=1)
    assert np.allclose(w, np.take_along_axis(full, idx.astype(np.int64), 1), rtol=1e-13)
    assert np.allclose(np.sort(w, axis=1)[:, ::-1], w)
    # no renorm, k < E: plain softmax probabilities of the selected experts
    idx2 = orc.topk_of_logits(logits, 2)
    w2 = orc.gate_weights(logits, idx2, renorm=False)
    assert np.allclose(w2, np.take_along_axis(full, idx2.astype(np.int64), 1), rtol=1e-13)
    assert (w2.sum(axis=1) < 1).all()
    # k = 1 with renorm: weight one
    idx1 = orc.topk_of_logits(logits, 1)
    assert np.allclose(orc.gate_weights(logits, idx1, True), 1.0)
    assert (idx1[:, 0] == logits.argmax(axis=1)).all()
    # all-equal logits: lowest ids, uniform weights
    flat = np.full((4, 6), 0.37)
    idxf = orc.topk_of_logits(flat, 3)
    assert (idxf == np.array([0, 1, 2])).all()
    assert np.allclose(orc.gate_weights(flat, idxf, True), 1.0 / 3)
    # a huge bias on one expert: it comes first and takes all the un-renormalised mass
    x = r.normal(size=(5, 4)); wr = r.normal(size=(6, 4))
    bias = np.zeros(6); bias[4] = 1e3
    idxb, wb, _ = orc.route_topk(x, wr, 2, bias, renorm=False)
    assert (idxb[:, 0] == 4).all() and np.allclose(wb[:, 0], 1.0) and np.allclose(wb[:, 1], 0.0)


def test_router_duplicate_rows_tie_to_lower_id():
    r = _rng(6)
    x = r.normal(size=(40, 33))
    wr = r.normal(size=(8, 33))
    wr[6] = wr[1]
    idx, w, logits = orc.route_topk(x, wr, 8)
    assert (logits[:, 6] == logits[:, 1]).all()
    for t in range(40):
        pos1 = idx[t].tolist().index(1)
        assert idx[t, pos1 + 1] == 6


# ---------------------------------------------------------------- permutation (a2)
def test_permute_against_library_and_invariants():
    r = _rng(7)
    T, k, E = 37, 3, 11
    idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    idx[np.isin(idx, [10])] = 0                            # expert 10 never used -> empty group
    counts, off, row_src, row_of = orc.permute(idx, E)
    flat = idx.reshape(-1)
    assert (counts == np.bincount(flat, minlength=E)).all()
    assert counts[10] == 0 and off[E] == T * k and off[0] == 0
    assert (np.diff(off) == counts).all()
    assert (row_src == np.argsort(flat, kind="stable")).all()
    assert (row_of[row_src] == np.arange(T * k)).all()
    assert (row_src[row_of] == np.arange(T * k)).all()
    for e in range(E):
        seg = row_src[off[e]:off[e + 1]]
        assert (flat[seg] == e).all()
        assert (np.diff(seg) > 0).all()
    tok = row_src // k
    assert (np.bincount(tok, minlength=T) == k).all()       # every token exactly k times
    x = r.normal(size=(T, 5))
    xp = orc.gather_rows(x, row_src, k)
    for rr in range(T * k):
        assert (xp[rr] == x[row_src[rr] // k]).all()


# ---------------------------------------------------------------- experts (a3)
def test_silu_pins():
    z = np.linspace(-30, 30, 241)
    assert orc.silu(np.array(0.0)) == 0.0
    assert np.allclose(orc.silu(z), z * scipy.special.expit(z), rtol=1e-14, atol=1e-300)
    assert np.allclose(orc.silu(z) - orc.silu(-z), z, rtol=1e-13, atol=1e-13)
    assert abs(orc.silu(np.array(40.0)) - 40.0) < 1e-12
    assert orc.silu(np.array(-1.0)) < 0


def test_expert_ffn_scalar_brute_force():
    p = _tiny_layer(8, d=3, f=4, E=1)
    v = p["x"][0]
    wg, wu, wd = p["wg"][0], p["wu"][0], p["wd"][0]
    import math
    want = []
    for j in range(3):
        acc = 0.0
        for i in range(4):
            g = sum(wg[i, c] * v[c] for c in range(3))
            u = sum(wu[i, c] * v[c] for c in range(3))
            acc += wd[j, i] * (g / (1.0 + math.exp(-g))) * u
        want.append(acc)
    assert np.allclose(orc.expert_ffn(v, wg, wu, wd), want, rtol=1e-13)


def test_grouped_single_expert_is_dense_swiglu_mlp_library():
    p = _tiny_layer(9, T=13, d=8, f=12, E=1)
    x = torch.from_numpy(p["x"])
    wg, wu, wd = (torch.from_numpy(p[n][0]) for n in ("wg", "wu", "wd"))
    ref = (torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)) @ wd.T
    got = orc.grouped_swiglu(p["x"], np.array([0, 13]), p["wg"], p["wu"], p["wd"])
    assert np.allclose(got, ref.numpy(), rtol=1e-12, atol=1e-14)


def test_grouped_rows_use_their_own_expert_and_empty_groups():
    p = _tiny_layer(10, T=9, d=4, f=6, E=4)
    off = np.array([0, 3, 3, 7, 9])                        # expert 1 is empty
    y = orc.grouped_swiglu(p["x"], off, p["wg"], p["wu"], p["wd"])
    for e in range(4):
        for rr in range(off[e], off[e + 1]):
            assert np.allclose(y[rr], orc.expert_ffn(p["x"][rr], p["wg"][e], p["wu"][e], p["wd"][e]),
                               rtol=1e-13)
    assert (orc.grouped_swiglu(np.zeros_like(p["x"]), off, p["wg"], p["wu"], p["wd"]) == 0).all()
    y2 = orc.grouped_swiglu(p["x"], off, p["wg"], p["wu"], 2.5 * p["wd"])
    assert np.allclose(y2, 2.5 * y, rtol=1e-13)


# ---------------------------------------------------------------- combine / whole layer (a4)
def test_combine_definition():
    r = _rng(11)
    T, k, d = 6, 3, 5
    y = r.normal(size=(T * k, d)); w = r.random(size=(T, k))
    row_of = r.permutation(T * k).astype(np.int32)
    out = orc.combine(y, row_of, w, T, k)
    for t in range(T):
        want = sum(w[t, s] * y[row_of[t * k + s]] for s in range(k))
        assert np.allclose(out[t], want, rtol=1e-14)


@pytest.mark.parametrize("k", [1, 2, 4])
def test_stepwise_pipeline_equals_brute_force(k):
    p = _tiny_layer(12 + k, T=23, d=8, f=12, E=6)
    a = orc.moe_layer_stepwise(p["x"], p["wr"], p["wg"], p["wu"], p["wd"], k)
    b = orc.moe_layer_brute_force(p["x"], p["wr"], p["wg"], p["wu"], p["wd"], k)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)


def test_identical_experts_invariant():
    """All experts equal + renormalised gates => out[t] = FFN(x[t]) whatever the routing."""
    p = _tiny_layer(20, T=17, d=8, f=12, E=5)
    for n in ("wg", "wu", "wd"):
        p[n] = np.repeat(p[n][:1], 5, axis=0)
    out = orc.moe_layer_stepwise(p["x"], p["wr"], p["wg"], p["wu"], p["wd"], 3, renorm=True)
    x = torch.from_numpy(p["x"])
    wg, wu, wd = (torch.from_numpy(p[n][0]) for n in ("wg", "wu", "wd"))
    ref = (torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)) @ wd.T
    assert np.allclose(out, ref.numpy(), rtol=1e-12, atol=1e-14)


def test_token_permutation_and_expert_relabelling_equivariance():
    p = _tiny_layer(21, T=19, d=8, f=12, E=6)
    base = orc.moe_layer_stepwise(p["x"], p["wr"], p["wg"], p["wu"], p["wd"], 2)
    perm_t = _rng(1).permutation(19)
    out_t = orc.moe_layer_stepwise(p["x"][perm_t], p["wr"], p["wg"], p["wu"], p["wd"], 2)
    assert np.allclose(out_t, base[perm_t], rtol=1e-12, atol=1e-14)
    perm_e = _rng(2).permutation(6)
    out_e = orc.moe_layer_stepwise(p["x"], p["wr"][perm_e], p["wg"][perm_e], p["wu"][perm_e],
                                   p["wd"][perm_e], 2)
    assert np.allclose(out_e, base, rtol=1e-12, atol=1e-14)


def test_config1_full_brute_force_vs_stepwise():
    cfg = synth.CONFIGS[1]
    L = synth.make_layer(cfg, "cpu", seed=1)
    a = {n: synth.to_f64(L[n]) for n in ("x", "w_router", "w_gate", "w_up", "w_down")}
    s = orc.moe_layer_stepwise(a["x"], a["w_router"], a["w_gate"], a["w_up"], a["w_down"], cfg.k)
    b = orc.moe_layer_brute_force(a["x"], a["w_router"], a["w_gate"], a["w_up"], a["w_down"], cfg.k)
    assert s.shape == (16, 256)
    assert np.allclose(s, b, rtol=1e-12, atol=1e-18)


# ---------------------------------------------------------------- stack helpers, by-products
def test_rmsnorm_against_library_and_closed_form():
    r = _rng(30)
    x = r.normal(size=(5, 16)); g = r.normal(size=16)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), eps=1e-5)
    assert np.allclose(orc.rmsnorm(x, g, 1e-5), ref.numpy(), rtol=1e-13)
    c = np.full((1, 8), 3.0)
    assert np.allclose(orc.rmsnorm(c, np.ones(8), 1e-5), 3.0 / np.sqrt(9.0 + 1e-5), rtol=1e-15)


def test_decoder_stack_is_prenorm_residual():
    p = _tiny_layer(31, T=5, d=8, f=12, E=4)
    layers = [dict(gain=np.ones(8), w_router=p["wr"], bias=None, w_gate=p["wg"], w_up=p["wu"],
                   w_down=p["wd"]) for _ in range(2)]
    h = orc.decoder_stack(p["x"], layers, 2)
    h1 = p["x"] + orc.moe_layer_brute_force(orc.rmsnorm(p["x"], np.ones(8)), p["wr"], p["wg"],
                                            p["wu"], p["wd"], 2)
    h2 = h1 + orc.moe_layer_brute_force(orc.rmsnorm(h1, np.ones(8)), p["wr"], p["wg"], p["wu"],
                                        p["wd"], 2)
    assert np.allclose(h, h2, rtol=1e-13)
    zero = [dict(gain=np.ones(8), w_router=p["wr"], bias=None, w_gate=p["wg"], w_up=p["wu"],
                 w_down=np.zeros_like(p["wd"]))]
    assert np.allclose(orc.decoder_stack(p["x"], zero, 2), p["x"])


def test_decoder_stack_with_identical_experts_is_a_dense_prenorm_mlp_stack():
    """If all experts of a layer share their weights, renormalised gates make the MoE block the
    plain FFN, so the stack is h <- h + Wd(silu(Wg n) * (Wu n)), n = rms_norm(h) * gain: written
    here with torch's own rms_norm / silu / linear in fp64, layer weights and gains all different."""
    F = torch.nn.functional
    g = torch.Generator().manual_seed(77)
    T, d, f, E, n_layers, eps = 7, 12, 20, 5, 3, 1e-5
    x = torch.randn(T, d, generator=g, dtype=torch.float64)
    layers, h = [], x.clone()
    for _ in range(n_layers):
        wg = torch.randn(f, d, generator=g, dtype=torch.float64) * 0.4
        wu = torch.randn(f, d, generator=g, dtype=torch.float64) * 0.4
        wd = torch.randn(d, f, generator=g, dtype=torch.float64) * 0.4
        gain = 1.0 + 0.3 * torch.randn(d, generator=g, dtype=torch.float64)
        wr = torch.randn(E, d, generator=g, dtype=torch.float64)
        layers.append(dict(gain=gain.numpy(), w_router=wr.numpy(), bias=None,
                           w_gate=np.stack([wg.numpy()] * E), w_up=np.stack([wu.numpy()] * E),
                           w_down=np.stack([wd.numpy()] * E)))
        n = F.rms_norm(h, (d,), weight=gain, eps=eps)
        h = h + F.linear(F.silu(F.linear(n, wg)) * F.linear(n, wu), wd)
    got = orc.decoder_stack(x.numpy(), layers, 2, True, eps)
    np.testing.assert_allclose(got, h.numpy(), rtol=1e-11, atol=1e-12)
    # the residual and the per-layer normalisation both matter: dropping either changes the result
    no_res = x.clone()
    for L in layers:
        n = F.rms_norm(no_res, (d,), weight=torch.from_numpy(L["gain"]), eps=eps)
        no_res = F.linear(F.silu(F.linear(n, torch.from_numpy(L["w_gate"][0]))) *
                          F.linear(n, torch.from_numpy(L["w_up"][0])), torch.from_numpy(L["w_down"][0]))
    assert np.abs(got - no_res.numpy()).max() > 1e-2


def test_skewness_quarter_is_rounded_up():
    """Hand values for expert counts not divisible by 4 (quarter = ceil(E/4) experts), and the
    lower bound 0.25 the paper states, for every E."""
    assert abs(orc.skewness(np.array([5, 4, 3, 2, 1, 0])) - 9 / 15) < 1e-15          # E = 6: 2 experts
    assert abs(orc.skewness(np.array([1, 9, 2, 8, 3, 7, 4, 6, 5, 0])) - 24 / 45) < 1e-15   # E = 10: 3
    assert abs(orc.skewness(np.array([2, 7, 1, 5, 3])) - 12 / 18) < 1e-15            # E = 5: 2
    assert orc.skewness(np.array([3.0])) == 1.0
    for E in range(1, 21):
        s = orc.skewness(np.full(E, 7))
        assert 0.25 <= s <= 1.0 and abs(s - (-(-E // 4)) / E) < 1e-15


def test_skewness_and_hot_experts():
    """Table I caption: skewness = share of pairs on the hottest quarter of experts, in [0.25, 1]."""
    assert orc.skewness(np.full(8, 10)) == 0.25
    assert orc.skewness(np.array([100, 0, 0, 0, 0, 0, 0, 0])) == 1.0
    assert abs(orc.skewness(np.array([4, 3, 2, 1])) - 0.4) < 1e-15
    assert orc.hot_experts(np.array([3, 9, 9, 1, 9]), 2).tolist() == [1, 2]
    assert orc.hot_experts(np.array([3, 9, 9, 1, 9]), 4).tolist() == [1, 2, 4, 0]


def test_config3_router_is_skewed_like_the_paper_describes():
    """Synthetic Zipf router: skewness inside the paper's range and far above uniform."""
    cfg = synth.CONFIGS[3]
    g = torch.Generator().manual_seed(5)
    x = (torch.randn(cfg.T, cfg.d_model, generator=g) * cfg.x_std).to(torch.bfloat16)
    wr = (torch.randn(cfg.E, cfg.d_model, generator=g) * cfg.router_std).to(torch.bfloat16)
    rank = torch.randperm(cfg.E, generator=g).float() + 1
    bias = (-cfg.zipf * torch.log(rank)).numpy()
    idx, w, _ = orc.route_topk(synth.to_f64(x), synth.to_f64(wr), cfg.k, bias, True)
    counts, *_ = orc.permute(idx, cfg.E)
    s = orc.skewness(counts)
    assert 0.5 < s <= 1.0
    assert counts.sum() == cfg.P


# ---------------------------------------------------------------- affinity / draft routing (n2)
def test_affinity_matches_library_pairwise_distance():
    """scipy's pairwise Euclidean distance on the experts' concatenated parameters."""
    from scipy.spatial.distance import cdist
    L = _tiny_layer(31, E=6)
    D = orc.affinity_table(L["wg"], L["wu"], L["wd"])
    flat = np.concatenate([L["wg"].reshape(6, -1), L["wu"].reshape(6, -1),
                           L["wd"].reshape(6, -1)], axis=1)
    np.testing.assert_allclose(D, cdist(flat, flat, metric="euclidean"), rtol=1e-12, atol=1e-12)


def test_affinity_metric_axioms_and_planted_values():
    L = _tiny_layer(32, E=5)
    # expert 4 := expert 1 (distance 0), expert 3 := expert 0 + constant 0.5 in every entry
    for k in ("wg", "wu", "wd"):
        L[k][4] = L[k][1]
        L[k][3] = L[k][0] + 0.5
    D = orc.affinity_table(L["wg"], L["wu"], L["wd"])
    n_param = L["wg"][0].size + L["wu"][0].size + L["wd"][0].size
    assert np.all(np.diag(D) == 0) and np.allclose(D, D.T)
    assert D[1, 4] == 0
    assert D[0, 3] == pytest.approx(0.5 * np.sqrt(n_param), rel=1e-12)
    for i, j, k in itertools.permutations(range(5), 3):
        assert D[i, j] <= D[i, k] + D[k, j] + 1e-9


def test_nearest_draft_expert_cases():
    D = np.array([[0, 5, 1, 7],
                  [5, 0, 3, 2],
                  [1, 3, 0, 3],
                  [7, 2, 3, 0]], dtype=np.float64)
    assert orc.nearest_draft_expert(D, [0, 1, 2, 3]).tolist() == [0, 1, 2, 3]      # all resident
    assert orc.nearest_draft_expert(D, [2]).tolist() == [2, 2, 2, 2]                # N = 1
    assert orc.nearest_draft_expert(D, [3, 0]).tolist() == [0, 3, 0, 3]            # by distance
    # expert 2 is equally far (3) from 1 and 3 -> lower id; order of draft_ids is irrelevant
    assert orc.nearest_draft_expert(D, [3, 1]).tolist() == [1, 1, 1, 3]
    assert orc.nearest_draft_expert(D, [1, 3]).tolist() == [1, 1, 1, 3]


def test_route_draft_reductions():
    L = _tiny_layer(33, T=40, E=6)
    D = orc.affinity_table(L["wg"], L["wu"], L["wd"])
    idx, w, _ = orc.route_topk(L["x"], L["wr"], 2)
    idx_all, w_all = orc.route_topk_draft(L["x"], L["wr"], 2, list(range(6)), D)
    assert np.array_equal(idx, idx_all) and np.array_equal(w, w_all)               # N = E
    draft = [4, 1, 2]
    idx_d, w_d = orc.route_topk_draft(L["x"], L["wr"], 2, draft, D)
    assert set(np.unique(idx_d)) <= set(draft) and np.array_equal(w_d, w)
    keep = np.isin(idx, draft)
    assert np.array_equal(idx_d[keep], idx[keep])                                  # residents stay
    for e_from, e_to in zip(idx[~keep], idx_d[~keep]):
        assert all(D[e_from, e_to] <= D[e_from, dd] for dd in draft)


def test_draft_layer_invariants():
    """Copies of a resident expert are replaced by that expert without changing the output;
    with every expert resident the draft layer is the target layer."""
    L = _tiny_layer(34, T=12, E=6)
    for k in ("wg", "wu", "wd"):
        L[k][3] = L[k][0]
        L[k][5] = L[k][2]
    D = orc.affinity_table(L["wg"], L["wu"], L["wd"])
    full = orc.moe_layer_stepwise(L["x"], L["wr"], L["wg"], L["wu"], L["wd"], 2)
    out_all = orc.moe_layer_draft(L["x"], L["wr"], L["wg"], L["wu"], L["wd"], 2, range(6), D)[0]
    np.testing.assert_allclose(out_all, full, rtol=1e-13, atol=1e-13)
    out_d, idx_d, _ = orc.moe_layer_draft(L["x"], L["wr"], L["wg"], L["wu"], L["wd"], 2,
                                          [0, 1, 2, 4], D)
    assert set(np.unique(idx_d)) <= {0, 1, 2, 4}
    np.testing.assert_allclose(out_d, full, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- sampling acceptance (n3)
def _one_hot(ids, V):
    p = np.zeros(ids.shape + (V,), dtype=np.float64)
    np.put_along_axis(p, ids[..., None].astype(np.int64), 1.0, axis=-1)
    return p


def test_accept_sample_reduces_to_greedy_on_one_hot():
    """Point-mass distributions: the rule keeps a draft iff it equals the target's token and
    redraws exactly the target's token -> the greedy rule (pinned to Fig. 4 above)."""
    r = _rng(41)
    B, gamma, V = 64, 5, 11
    draft = r.integers(0, V, size=(B, gamma)).astype(np.int32)
    target = r.integers(0, V, size=(B, gamma + 1)).astype(np.int32)
    agree = r.random(size=(B, gamma)) < 0.7
    target[:, :gamma] = np.where(agree, draft, target[:, :gamma])
    alen_g, out_g = orc.accept(draft, target)
    alen_s, out_s = orc.accept_sample(draft, _one_hot(draft, V), _one_hot(target, V),
                                      r.random(size=(B, gamma)), r.random(size=B))
    assert np.array_equal(alen_g, alen_s) and np.array_equal(out_g, out_s)
    g = _read_golden("fig4_accept.txt")
    d1, t1 = np.array([g["draft"]]), np.array([g["target"]])
    a1, o1 = orc.accept_sample(d1, _one_hot(d1, 40000), _one_hot(t1, 40000),
                               np.full((1, 5), 0.5), np.array([0.5]))
    assert a1[0] == g["generated"][0] and o1[0].tolist() == g["out_tokens"]


def test_accept_sample_identical_distributions_keep_everything():
    r = _rng(42)
    B, gamma, V = 16, 4, 9
    p = r.random(size=(B, gamma + 1, V)); p /= p.sum(-1, keepdims=True)
    draft = r.integers(0, V, size=(B, gamma)).astype(np.int32)
    alen, out = orc.accept_sample(draft, p[:, :gamma], p, r.random(size=(B, gamma)), r.random(size=B))
    assert np.all(alen == gamma + 1) and np.array_equal(out[:, :gamma], draft)
    assert np.all((out[:, gamma] >= 0) & (out[:, gamma] < V))


def test_accept_sample_emits_the_target_distribution():
    """The theorem behind the rule: with the draft token drawn from pd, the FIRST emitted
    token is distributed exactly as pt, and the draft is kept with probability
    sum_v min(pd, pt).  Monte Carlo over 2*10^5 sequences, V = 6."""
    r = _rng(43)
    V, B = 6, 200000
    pd = np.array([0.05, 0.30, 0.10, 0.25, 0.20, 0.10])
    pt = np.array([0.25, 0.05, 0.10, 0.15, 0.05, 0.40])
    draft = r.choice(V, size=(B, 1), p=pd).astype(np.int32)
    p_draft = np.broadcast_to(pd, (B, 1, V))
    p_target = np.broadcast_to(pt, (B, 2, V))
    alen, out = orc.accept_sample(draft, p_draft, p_target, r.random(size=(B, 1)), r.random(size=B))
    freq = np.bincount(out[:, 0], minlength=V) / B
    sigma = np.sqrt(pt * (1 - pt) / B)
    assert np.all(np.abs(freq - pt) < 4.5 * sigma), (freq, pt)
    keep = np.mean(alen == 2)
    want = np.minimum(pd, pt).sum()
    assert abs(keep - want) < 4.5 * np.sqrt(want * (1 - want) / B)
    # after a kept draft the extra token follows pt as well
    f2 = np.bincount(out[alen == 2, 1], minlength=V) / np.sum(alen == 2)
    assert np.all(np.abs(f2 - pt) < 5 * np.sqrt(pt * (1 - pt) / np.sum(alen == 2)))


def test_accept_sample_inverse_cdf_boundaries():
    """Draws by hand: residual (pt - pd)+ = [0, .2, 0, .3] -> u < .4 gives id 1, else id 3."""
    pd = np.array([[[0.5, 0.1, 0.4, 0.0]]])
    pt = np.array([[[0.2, 0.3, 0.2, 0.3], [0.25, 0.25, 0.25, 0.25]]])
    draft = np.array([[0]], dtype=np.int32)
    # u*pd = u*0.5 < 0.2  <=> u < 0.4 keeps the draft
    a, o = orc.accept_sample(draft, pd, pt, np.array([[0.39]]), np.array([0.6]))
    assert a[0] == 2 and o[0].tolist() == [0, 2]          # kept; extra token: cdf .25 .5 .75 1
    a, o = orc.accept_sample(draft, pd, pt, np.array([[0.41]]), np.array([0.39]))
    assert a[0] == 1 and o[0].tolist() == [1, -1]
    a, o = orc.accept_sample(draft, pd, pt, np.array([[0.41]]), np.array([0.40]))
    assert a[0] == 1 and o[0].tolist() == [3, -1]
    a, o = orc.accept_sample(draft, pd, pt, np.array([[0.99]]), np.array([0.0]))
    assert o[0].tolist() == [1, -1]                        # zero-weight id 0 is never drawn


# ---------------------------------------------------------------- reporting helpers (n4)
def test_greedy_tokens_is_first_occurrence_argmax():
    r = _rng(51)
    logits = r.integers(-3, 4, size=(200, 17)).astype(np.float64)     # many exact ties
    assert np.array_equal(orc.greedy_tokens(logits), np.argmax(logits, axis=1))
    assert orc.greedy_tokens(np.array([[1.0, 5.0, 5.0, 2.0]])).tolist() == [1]


def test_active_expert_bytes_and_speedup_model():
    assert orc.active_expert_bytes([3, 0, 1, 0], 100) == 200
    # Mixtral-shaped block: 3*d*f*2 bytes per expert; Table I lists 8 experts per block
    assert orc.active_expert_bytes([1] * 8, 3 * 4096 * 14336 * 2) == 2818572288
    # Eq. 1 is Eq. 2 at lambda = 1; a free draft model (c = 0) yields tau itself; with
    # i.i.d. acceptance 0.7 and gamma = 4, tau = (1 - 0.7^5) / 0.3
    tau = (1 - 0.7 ** 5) / 0.3
    assert orc.expected_speedup(tau, 4, 0.0) == pytest.approx(2.7731, abs=1e-4)
    assert orc.expected_speedup(tau, 4, 0.1, 1.0) == pytest.approx(tau / 1.4)
    # Sec. 3.3's examples: gamma = 8 with lambda ~ 6 (B = 1) against lambda ~ 2 (B = 32):
    # the larger batch triples-or-so the speed-up for a cheap draft model
    s1, s32 = orc.expected_speedup(4.0, 8, 0.05, 6.0), orc.expected_speedup(4.0, 8, 0.05, 2.0)
    assert s32 / s1 == pytest.approx(6.4 / 2.4)
