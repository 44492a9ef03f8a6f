"""Why the floating-point parity bar is measured per output row against the row's largest
magnitude.  A CPU model of the rounding points any bf16 matrix-core implementation has (h
rounded to bf16 before the second contraction, y_perm and out rounded to bf16 once each)
applied to the ORACLE's own fp64 intermediates: it shows the error level the arithmetic
itself allows, independent of any kernel."""
import numpy as np
import torch

from oracle import moe_verify_oracle as orc
from workloads.metrics import floored_rel_err


def _bf16(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16) \
        .to(torch.float64).numpy()


def _row_err(got, want):
    return float((np.abs(got - want).max(axis=1) / np.abs(want).max(axis=1)).max())


def test_mandatory_bf16_roundings_fit_row_norm_bar_but_not_elementwise_floor():
    rng = np.random.default_rng(0)
    T, d, f, E, k = 96, 512, 1024, 4, 2
    x = _bf16(rng.normal(size=(T, d)) / np.sqrt(d))
    wr = _bf16(rng.normal(size=(E, d)) * 0.02)
    wg = _bf16(rng.normal(size=(E, f, d)) * 0.02)
    wu = _bf16(rng.normal(size=(E, f, d)) * 0.02)
    wd = _bf16(rng.normal(size=(E, d, f)) * 0.02)
    want = orc.moe_layer_brute_force(x, wr, wg, wu, wd, k)

    idx, w, _ = orc.route_topk(x, wr, k)
    got = np.zeros_like(want)
    for t in range(T):
        acc = np.zeros(d)
        for s in range(k):
            e = idx[t, s]
            h = _bf16(orc.silu(wg[e] @ x[t]) * (wu[e] @ x[t]))       # rounding point 1
            y = _bf16(wd[e] @ h)                                     # rounding point 2
            acc += np.float32(w[t, s]) * y
        got[t] = _bf16(acc)                                          # rounding point 3
    row = _row_err(got, want)
    elem = floored_rel_err(got, want, floor_frac=1e-3)
    rms = float((np.sqrt(((got - want) ** 2).mean(axis=1)) / np.sqrt((want ** 2).mean(axis=1))).max())
    print(f"ideal bf16 pipeline: per-row err {row:.2e}, per-row rms err {rms:.2e}, "
          f"floored element-wise err {elem:.2e}")
    # second bar of the GPU tests: per-row rms error <= 5e-3.  Unbiased rounding stays below it
    # with margin; a 1 % systematic error (which the max-norm bar alone would pass) does not.
    assert rms < 4e-3, rms
    biased = got * 1.01
    assert float((np.sqrt(((biased - want) ** 2).mean(axis=1)) /
                  np.sqrt((want ** 2).mean(axis=1))).min()) > 5e-3
    # the per-row max-norm error of an ideal implementation sits below the 1e-2 bar ...
    assert row < 1e-2, row
    # ... while element-wise relative error with a floor at 1e-3 of the tensor maximum is
    # already beyond 1e-2 for it: small elements inherit the absolute rounding error of h.
    assert elem > 1e-2, elem


def test_fp32_arithmetic_meets_row_bar_but_not_the_floored_elementwise_one():
    """fp32 mode on the cfg-1 shape, no kernel involved: the same definition evaluated with
    fp32 products and fp32 running sums (numpy float32 matmuls; h and y rounded to fp32).
    Accumulated round-off is a few 1e-7 of a row's typical magnitude, so the per-row max-norm
    error is far below 1e-5, while an element 1000 times smaller than the tensor maximum sees
    that same absolute error 1000 times larger in relative terms: the element-wise measure
    floored at 1e-3 of the maximum cannot reach 1e-5 in fp32 arithmetic.  The GPU tests
    therefore assert the floored measure at 1e-3 (and print it), the row measure at 1e-5."""
    rng = np.random.default_rng(1)
    T, d, f, E, k = 64, 256, 512, 8, 2
    f32 = np.float32
    x = (rng.normal(size=(T, d)) * 0.02).astype(f32)
    wr = (rng.normal(size=(E, d)) * 0.1).astype(f32)
    wg = (rng.normal(size=(E, f, d)) * 0.02).astype(f32)
    wu = (rng.normal(size=(E, f, d)) * 0.02).astype(f32)
    wd = (rng.normal(size=(E, d, f)) * 0.02).astype(f32)
    w64 = [a.astype(np.float64) for a in (x, wr, wg, wu, wd)]
    want = orc.moe_layer_brute_force(*w64, k)
    idx, w, _ = orc.route_topk(w64[0], w64[1], k)
    got = np.zeros((T, d), dtype=f32)
    for t in range(T):
        for s in range(k):
            e = idx[t, s]
            g = wg[e] @ x[t]
            h = (g / (f32(1) + np.exp(-g))) * (wu[e] @ x[t])
            got[t] += f32(w[t, s]) * (wd[e] @ h)
    row = _row_err(got.astype(np.float64), want)
    elem = floored_rel_err(got.astype(np.float64), want, floor_frac=1e-3)
    print(f"fp32 arithmetic: per-row err {row:.2e}, floored element-wise err {elem:.2e}")
    assert row < 1e-5, row
    assert 1e-5 < elem < 1e-3, elem
