"""Plain fp64 CPU definition of the MoE verification layer and the greedy acceptance check.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and the
`cpu_baseline` leg of the benchmark may import it.  It shares no code, table or constant
with the HIP library; it is numpy only, fp64 throughout, written to be checked against the
paper by eye, not to be fast.

What the paper fixes (SpecMoE, arxiv 2604.10152):

* Sec. 2.1 "Sparsely activated MoE block" and Fig. 1(b): an MoE block is a gate function
  plus E experts, each the size of the FFN layer; the gate picks the top-K experts of every
  token and only those run; their outputs are mixed by the gate.
* Sec. 2.2 "Algorithm" and Fig. 4: at verification time the target model scores all draft
  tokens of all sequences in parallel and emits one extra token per sequence, so the layer
  sees T = B*(gamma+1) tokens at once.
* Sec. 4 "SpecMoE configuration" and the caption of Fig. 4: greedy verification keeps the
  draft tokens that match the target's greedy tokens exactly, discards the first mismatch
  and everything after it, and appends the target's own token at that position.
* Sec. 3.2 "Expert replacement policy": expert activations are counted during verification.

What the paper leaves open and this file reads as follows:

* gate = linear router (+ optional per-expert bias), softmax over all E logits, selection
  of the k largest LOGITS (ties go to the lower expert id, slots ordered by descending
  logit then ascending id), gate weights = softmax probabilities at the selected ids,
  optionally renormalised to sum to one;
* expert = bias-free SwiGLU FFN:  FFN_e(v) = Wd_e ( silu(Wg_e v) * (Wu_e v) ),
  silu(z) = z / (1 + exp(-z));
* no capacity limit: every token is served by exactly k experts;
* the permutation by expert is stable (ascending flat pair index t*k+s inside an expert);
* accept_len counts the accepted drafts plus the one token the target contributes.

Pins (tests/test_oracle_pins.py): the worked example of Fig. 4 (5 drafts, mismatch at the
4th -> 3 accepted, 4 generated), the geometric closed form of the mean acceptance length,
exhaustive match patterns, softmax-over-selected closed form, k=E / k=1 / all-equal /
one-hot special cases, a stable library argsort, bincount, dense-MLP reduction for E=1,
identical-experts invariant, token-permutation and expert-relabelling equivariance, and
brute force per token against the step-wise (route, permute, grouped, combine) pipeline.
The speculation-phase functions (affinity table, nearest draft expert, draft routing), the
sampling-based acceptance rule and the reporting helpers at the end of the file are pinned in
the same test file: a library pairwise-distance routine, metric axioms and planted
duplicates; reduction of the sampling rule to the greedy one on one-hot distributions, the
"emitted token is distributed as the target" theorem and the sum-of-minima acceptance rate
by Monte Carlo; numpy's first-occurrence argmax; the speed-up numbers the paper's own
examples imply.  No function in this file is unpinned.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# a1  router: logits, top-k on logits, softmax gate weights          (Sec. 2.1, Fig. 1b)
# --------------------------------------------------------------------------------------
def router_logits(x, w_router, bias=None):
    """l[t,e] = bias[e] + sum_j x[t,j] * Wr[e,j]   in fp64.

    Every expert column is produced by the same matrix-vector routine, so two experts with
    identical router rows get bit-identical logits (ties are then decided by expert id).
    """
    x = np.asarray(x, dtype=F64)
    w_router = np.asarray(w_router, dtype=F64)
    T, E = x.shape[0], w_router.shape[0]
    logits = np.empty((T, E), dtype=F64)
    for e in range(E):
        logits[:, e] = x @ w_router[e]
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=F64)[None, :]
    return logits


def topk_of_logits(logits, k):
    """idx[t,0..k-1]: the k experts with the largest logits of token t.

    Order of the slots: larger logit first; equal logits: lower expert id first.
    """
    logits = np.asarray(logits, dtype=F64)
    T, E = logits.shape
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    idx = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        ranked = sorted(range(E), key=lambda e: (-logits[t, e], e))
        idx[t, :] = ranked[:k]
    return idx


def gate_weights(logits, idx, renorm=True):
    """w[t,s] = softmax(l[t,:])[idx[t,s]], divided by its sum over s if `renorm`."""
    logits = np.asarray(logits, dtype=F64)
    m = logits.max(axis=1, keepdims=True)
    ex = np.exp(logits - m)
    p = ex / ex.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return w


def route_topk(x, w_router, k, bias=None, renorm=True):
    """Router of one MoE block: returns (idx int32 [T,k], w fp64 [T,k], logits fp64 [T,E])."""
    logits = router_logits(x, w_router, bias)
    idx = topk_of_logits(logits, k)
    w = gate_weights(logits, idx, renorm)
    return idx, w, logits


# --------------------------------------------------------------------------------------
# a2  grouping of the (token, slot) pairs by expert                   (Fig. 2; Sec. 3.2)
# --------------------------------------------------------------------------------------
def permute(idx, E):
    """Stable grouping of the P = T*k pairs by expert.

    Returns
      counts[E]            number of pairs routed to each expert (the activation counters)
      expert_offsets[E+1]  exclusive prefix sum of counts; rows of expert e are
                           [offsets[e], offsets[e+1])
      row_src[P]           sorted row r holds flat pair  row_src[r] = t*k + s
      row_of[P]            inverse:  row_of[t*k+s] = r
    Inside an expert the rows keep ascending flat pair index.
    """
    idx = np.asarray(idx)
    T, k = idx.shape
    P = T * k
    flat = idx.reshape(P)
    counts = np.zeros(E, dtype=np.int32)
    for p in range(P):
        counts[flat[p]] += 1
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    cursor = offsets[:E].copy()
    row_src = np.empty(P, dtype=np.int32)
    row_of = np.empty(P, dtype=np.int32)
    for p in range(P):                      # ascending flat index => stable
        e = flat[p]
        r = cursor[e]
        cursor[e] += 1
        row_src[r] = p
        row_of[p] = r
    return counts, offsets, row_src, row_of


def gather_rows(x, row_src, k):
    """x_perm[r] = x[row_src[r] // k]  (the token of pair row_src[r])."""
    x = np.asarray(x)
    return x[np.asarray(row_src, dtype=np.int64) // k]


# --------------------------------------------------------------------------------------
# a3  experts                                                                (Sec. 2.1)
# --------------------------------------------------------------------------------------
def silu(z):
    return z / (1.0 + np.exp(-z))


def expert_ffn(v, wg, wu, wd):
    """FFN_e(v) = Wd ( silu(Wg v) * (Wu v) ) for one vector or a stack of row vectors.

    v: [d] or [m,d];  wg, wu: [f,d];  wd: [d,f].  fp64.
    """
    v = np.asarray(v, dtype=F64)
    g = v @ np.asarray(wg, dtype=F64).T
    u = v @ np.asarray(wu, dtype=F64).T
    h = silu(g) * u
    return h @ np.asarray(wd, dtype=F64).T


def grouped_swiglu(x_perm, expert_offsets, w_gate, w_up, w_down):
    """y_perm[r] = FFN_e(x_perm[r]) for r in [offsets[e], offsets[e+1]), every expert e."""
    x_perm = np.asarray(x_perm, dtype=F64)
    E = len(expert_offsets) - 1
    y = np.zeros((x_perm.shape[0], np.asarray(w_down[0]).shape[0]), dtype=F64)
    for e in range(E):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi > lo:
            y[lo:hi] = expert_ffn(x_perm[lo:hi], w_gate[e], w_up[e], w_down[e])
    return y


# --------------------------------------------------------------------------------------
# a4  gate-weighted mix of the selected experts' outputs              (Sec. 2.1, Fig. 1b)
# --------------------------------------------------------------------------------------
def combine(y_perm, row_of, w, T, k):
    """out[t] = sum_s w[t,s] * y_perm[row_of[t*k+s]]."""
    y_perm = np.asarray(y_perm, dtype=F64)
    w = np.asarray(w, dtype=F64)
    out = np.zeros((T, y_perm.shape[1]), dtype=F64)
    for t in range(T):
        for s in range(k):
            out[t] += w[t, s] * y_perm[row_of[t * k + s]]
    return out


def moe_layer_stepwise(x, w_router, w_gate, w_up, w_down, k, bias=None, renorm=True):
    """The layer as the four steps route -> permute -> grouped experts -> combine."""
    x = np.asarray(x, dtype=F64)
    E = np.asarray(w_router).shape[0]
    idx, w, _ = route_topk(x, w_router, k, bias, renorm)
    _, offsets, row_src, row_of = permute(idx, E)
    x_perm = gather_rows(x, row_src, k)
    y_perm = grouped_swiglu(x_perm, offsets, w_gate, w_up, w_down)
    return combine(y_perm, row_of, w, x.shape[0], k)


def moe_layer_brute_force(x, w_router, w_gate, w_up, w_down, k, bias=None, renorm=True):
    """The definition, token by token:  out[t] = sum_s w[t,s] * FFN_{idx[t,s]}(x[t]).

    No grouping, no permutation.  `w_gate`, `w_up`, `w_down` are indexable by expert id
    (arrays [E,...] or lists); only the experts a token selects are touched.
    """
    x = np.asarray(x, dtype=F64)
    idx, w, _ = route_topk(x, w_router, k, bias, renorm)
    d_out = np.asarray(w_down[0]).shape[0]
    out = np.zeros((x.shape[0], d_out), dtype=F64)
    for t in range(x.shape[0]):
        for s in range(k):
            e = int(idx[t, s])
            out[t] += w[t, s] * expert_ffn(x[t], w_gate[e], w_up[e], w_down[e])
    return out


# --------------------------------------------------------------------------------------
# a5  greedy acceptance                      (Sec. 2.2 Fig. 4; Sec. 4 SpecMoE configuration)
# --------------------------------------------------------------------------------------
def accept(draft, target):
    """Greedy verification of gamma draft tokens per sequence.

    draft[b,i]  (i < gamma)   token the draft model proposed at position i
    target[b,i] (i <= gamma)  target model's greedy token at the same position; target[b,gamma]
                              is the extra token available when every draft matched
    n_b = number of leading positions with draft == target.  The first mismatching draft and
    everything after it are dropped and the target's token at that position is appended:
      accept_len[b] = n_b + 1                 (tokens generated this step, in [1, gamma+1])
      out_tokens[b, 0..n_b] = target[b, 0..n_b],  remaining entries -1
    """
    draft = np.asarray(draft)
    target = np.asarray(target)
    B, gamma = draft.shape
    if target.shape != (B, gamma + 1):
        raise ValueError("target must be [B, gamma+1]")
    accept_len = np.zeros(B, dtype=np.int32)
    out_tokens = np.full((B, gamma + 1), -1, dtype=np.int32)
    for b in range(B):
        n = 0
        while n < gamma and draft[b, n] == target[b, n]:
            n += 1
        accept_len[b] = n + 1
        for i in range(n + 1):
            out_tokens[b, i] = target[b, i]
    return accept_len, out_tokens


# --------------------------------------------------------------------------------------
# helpers for the multi-layer configuration (not in the paper: benchmark configuration 5)
# --------------------------------------------------------------------------------------
def rmsnorm(x, gain, eps=1e-5):
    """x / sqrt(mean(x^2) + eps) * gain, row-wise, fp64."""
    x = np.asarray(x, dtype=F64)
    ms = (x * x).mean(axis=1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, dtype=F64)[None, :]


def decoder_stack(x, layers, k, renorm=True, eps=1e-5):
    """h_0 = x;  h_{l+1} = h_l + MoE_l(RMSNorm_l(h_l)).

    `layers` is an iterable of dicts with keys gain, w_router, bias (or None), w_gate, w_up,
    w_down; it may be a generator so that layer weights are streamed.
    """
    h = np.asarray(x, dtype=F64)
    for layer in layers:
        n = rmsnorm(h, layer["gain"], eps)
        h = h + moe_layer_brute_force(n, layer["w_router"], layer["w_gate"], layer["w_up"],
                                      layer["w_down"], k, layer.get("bias"), renorm)
    return h


# --------------------------------------------------------------------------------------
# by-products used by the paper's policy and reporting
# --------------------------------------------------------------------------------------
def skewness(counts):
    """Share of routed pairs that go to the hottest quarter of the experts (Table I caption).

    The quarter is ceil(E / 4) experts: Sec. 6.1 states that the value lies between 0.25 and 1,
    which for E not divisible by 4 holds only if the quarter is rounded up (uniform counts then
    give ceil(E/4)/E >= 0.25).
    """
    counts = np.sort(np.asarray(counts, dtype=F64))[::-1]
    top = -(-len(counts) // 4)
    total = counts.sum()
    return float(counts[:top].sum() / total) if total > 0 else 0.0


def hot_experts(counts, n):
    """The n most activated experts of a block, ties to the lower id (Sec. 3.2 replacement)."""
    counts = np.asarray(counts)
    ranked = sorted(range(len(counts)), key=lambda e: (-int(counts[e]), e))
    return np.asarray(ranked[:n], dtype=np.int32)


# --------------------------------------------------------------------------------------
# n2  speculation phase: affinity table, nearest draft expert, draft routing   (Sec. 3.2)
# --------------------------------------------------------------------------------------
def affinity_table(w_gate, w_up, w_down):
    """D[i,j] = L2 distance between the parameters of experts i and j (Sec. 3.2,
    "Affinity-based expert selection mechanism": similarity of all expert pairs by L2
    distance, computed once, offline).

    Reading: an expert's parameters are its three matrices taken together, so
    D[i,j]^2 = |Wg_i - Wg_j|_F^2 + |Wu_i - Wu_j|_F^2 + |Wd_i - Wd_j|_F^2.
    """
    E = len(w_gate)
    D = np.zeros((E, E), dtype=F64)
    for i in range(E):
        for j in range(E):
            sq = 0.0
            for W in (w_gate, w_up, w_down):
                diff = np.asarray(W[i], dtype=F64) - np.asarray(W[j], dtype=F64)
                sq += float(np.sum(diff * diff))
            D[i, j] = np.sqrt(sq)
    return D


def nearest_draft_expert(affinity, draft_ids):
    """remap[e] = e if e is a draft expert, else the draft expert closest to e in the affinity
    table (Fig. 8b); equal distances go to the lower expert id."""
    affinity = np.asarray(affinity)
    E = affinity.shape[0]
    draft = [int(d) for d in draft_ids]
    remap = np.zeros(E, dtype=np.int32)
    for e in range(E):
        if e in draft:
            remap[e] = e
        else:
            remap[e] = min(draft, key=lambda dd: (affinity[e, dd], dd))
    return remap


def route_topk_draft(x, w_router, k, draft_ids, affinity, bias=None, renorm=True):
    """Speculation-phase routing (Sec. 3.2): the target's gate is used as it is; a selected
    expert that is not resident is replaced by its nearest draft expert.

    Readings: the replacement is per slot and keeps the slot's gate weight; two slots of a
    token may end up on the same draft expert (their weights then simply add in the mix).
    """
    idx, w, _ = route_topk(x, w_router, k, bias, renorm)
    remap = nearest_draft_expert(affinity, draft_ids)
    return remap[idx].astype(np.int32), w


def moe_layer_draft(x, w_router, w_gate, w_up, w_down, k, draft_ids, affinity, bias=None,
                    renorm=True):
    """The MoE block as the draft model runs it: only draft experts compute (Sec. 3.2)."""
    x = np.asarray(x, dtype=F64)
    T, E = x.shape[0], len(w_gate)
    idx, w = route_topk_draft(x, w_router, k, draft_ids, affinity, bias, renorm)
    _, offsets, row_src, row_of = permute(idx, E)
    y_perm = grouped_swiglu(gather_rows(x, row_src, k), offsets, w_gate, w_up, w_down)
    return combine(y_perm, row_of, w, T, k), idx, w


# --------------------------------------------------------------------------------------
# n3  sampling-based verification   (Sec. 6.3: the rule of the speculative-sampling method
#     the paper cites; temperature 1, so the probabilities are the models' softmax outputs)
# --------------------------------------------------------------------------------------
def _inverse_cdf(weights, u):
    """Smallest id v with  sum_{v' <= v} weights[v'] > u * sum(weights)   (ids in order)."""
    c = np.cumsum(np.asarray(weights, dtype=F64))
    v = int(np.searchsorted(c, u * c[-1], side="right"))
    return min(v, len(c) - 1)


def accept_sample(draft, p_draft, p_target, u_accept, u_sample):
    """Per sequence: draft token i (id x) is kept when u_accept[b,i] < min(1, pt(x)/pd(x)),
    tested as u*pd(x) < pt(x); at the first rejection the token is redrawn from the
    normalised positive part of (pt - pd) and everything after it is dropped; if all gamma
    drafts are kept, one more token is drawn from the target's distribution at position
    gamma.  Draws use the caller's uniforms u_sample[b] through the inverse CDF in id order.

    draft [B,gamma] ids; p_draft [B,gamma,V]; p_target [B,gamma+1,V]; u_* in [0,1).
    Returns accept_len [B] (kept drafts + 1) and out_tokens [B,gamma+1] padded with -1.
    """
    draft = np.asarray(draft)
    p_draft = np.asarray(p_draft, dtype=F64)
    p_target = np.asarray(p_target, dtype=F64)
    B, gamma = draft.shape
    accept_len = np.zeros(B, dtype=np.int32)
    out = np.full((B, gamma + 1), -1, dtype=np.int32)
    for b in range(B):
        n = gamma
        for i in range(gamma):
            xid = int(draft[b, i])
            if not (F64(u_accept[b, i]) * p_draft[b, i, xid] < p_target[b, i, xid]):
                n = i
                break
        out[b, :n] = draft[b, :n]
        if n < gamma:
            resid = np.maximum(p_target[b, n] - p_draft[b, n], 0.0)
            if resid.sum() <= 0.0:          # identical distributions cannot reject; guard only
                resid = p_target[b, n]
            out[b, n] = _inverse_cdf(resid, F64(u_sample[b]))
        else:
            out[b, n] = _inverse_cdf(p_target[b, gamma], F64(u_sample[b]))
        accept_len[b] = n + 1
    return accept_len, out


# --------------------------------------------------------------------------------------
# n4  reporting helpers
# --------------------------------------------------------------------------------------
def greedy_tokens(logits):
    """Greedy decoding (Sec. 4 "SpecMoE configuration"): the id of the largest logit per row,
    the lower id on ties."""
    logits = np.asarray(logits)
    out = np.zeros(logits.shape[0], dtype=np.int32)
    for r in range(logits.shape[0]):
        best = 0
        for v in range(1, logits.shape[1]):
            if logits[r, v] > logits[r, best]:
                best = v
        out[r] = best
    return out


def active_expert_bytes(counts, bytes_per_expert):
    """Parameter bytes of the experts that at least one token activated: the volume an
    offloading system would have to bring to the GPU for this block (Sec. 2.1 "Challenges",
    Fig. 3b) and the volume this build reads from HBM."""
    return int(np.count_nonzero(np.asarray(counts) > 0)) * int(bytes_per_expert)


def expected_speedup(tau, gamma, c, lam=1.0):
    """Eq. 1 (lam = 1) and Eq. 2:  S = tau / (gamma * c + lam)."""
    return F64(tau) / (F64(gamma) * F64(c) + F64(lam))
