"""CPU tests of the bf16 error model of the matrix-core path (tests/bf16_error_model.py) and of the bounds the GPU
parity tests take from it (tests/parity_metrics.py).  Nothing here needs a GPU.

What is shown:
 * the model is the oracle: with every rounding switched off it reproduces fwd_dense / bwd_dense to 1e-12, for windows
   that are and are not tile multiples (so its split into stored states and directly formed pairs is neutral);
 * its rounding routine is round-to-nearest-even to bf16 (against torch's conversion);
 * storing the exact gradient as bf16, with no other error, already exceeds "worst element <= 2e-2 of RMS(ref)":
   gradient tensors reach 10 x their RMS and half a bf16 ulp there is 4e-2 of the RMS - the stored value's own
   rounding has to be taken off before an element is judged;
 * with bf16 operands at the kernels' rounding points the error is RMS(err)/RMS(ref) = 2.5e-3 .. 3.6e-3 and the worst
   element (beyond its own storage rounding) stays below 5e-2 of RMS(ref) but exceeds 2e-2 of it on a third of the tensors or more:
   the GPU bounds (5e-3 RMS, 8e-2 worst element, and 1.2 x / 2 x the model on the same input) follow from these
   figures, and the 2e-2-of-RMS figure is out of reach for bf16 matrix-core operands;
 * the output error of the forward stays within max-abs 2e-2 beyond storage rounding.
"""
import math

import numpy as np
import pytest
import torch

from oracle import rattn_oracle as orc
from paper_2506_15545_amd import synth
import bf16_error_model as em
import parity_metrics as pm


def np64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def inputs(B, T, Hq, Hkv, seed, gains, std=1.0):
    x = synth.make_random_layer(B, T, Hq, Hkv, 128, "bf16", seed, std=std, with_dO=True, with_gains=gains)
    kw = dict(gamma_swa=np64(x["gamma_swa"]), gamma_rla=np64(x["gamma_rla"])) if gains else {}
    return [np64(x[n]) for n in ("q", "k", "v", "dO")], kw


def test_bf16_round_is_round_to_nearest_even():
    g = torch.Generator().manual_seed(3)
    x = torch.randn(20000, generator=g, dtype=torch.float64) * torch.exp(4 * torch.randn(20000, generator=g, dtype=torch.float64))
    ties = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, 2.0 ** -130], dtype=torch.float64)
    x = torch.cat([x, ties])
    want = x.to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(em.bf16_round(x.numpy()), want)
    # half an ulp really bounds the rounding error, and is attained at ties
    e = np.abs(em.bf16_round(x.numpy()) - x.numpy())
    assert np.all(e <= pm.half_ulp_bf16(x.numpy()) * (1 + 1e-12) + 1e-45)
    assert abs(em.bf16_round(1.0 + 2.0 ** -8) - (1.0 + 2.0 ** -8)) == pm.half_ulp_bf16(1.0)


@pytest.mark.parametrize("B,T,Hq,Hkv,W,gains,fm", [(1, 384, 4, 2, 128, True, "softmax"), (2, 256, 2, 1, 100, False, "softmax"),
                                                  (1, 512, 3, 1, 65, True, "relu"), (1, 256, 2, 2, 300, False, "softmax"),
                                                  (1, 640, 2, 1, 513, False, "softmax")])
def test_model_without_rounding_is_the_oracle(B, T, Hq, Hkv, W, gains, fm):
    (q, k, v, dO), kw = inputs(B, T, Hq, Hkv, 40 + T + W, gains)
    scale = 1 / math.sqrt(128)
    m = em.model_fwd_bwd(q, k, v, dO, W, scale=scale, exact=em.ROUNDING_POINTS, feature_map=fm, **kw)
    f = orc.fwd_dense(q, k, v, W, scale=scale, feature_map=fm, **kw)
    b = orc.bwd_dense(q, k, v, dO, W, scale=scale, feature_map=fm, **kw)
    for n, ref in (("o", f["o"]), ("xs", f["xs"]), ("xr", f["xr"]), ("dq", b["dq"]), ("dk", b["dk"]), ("dv", b["dv"])):
        scale_n = max(1.0, float(np.abs(ref).max()))
        assert float(np.abs(m[n] - ref).max()) <= 1e-11 * scale_n, n


SWEEP = [  # B, T, Hq, Hkv, W, gains, seed
    (1, 128, 6, 1, 192, True, 95119), (3, 128, 6, 1, 62, False, 488218), (1, 256, 12, 2, 46, False, 442182),
    (1, 384, 6, 2, 300, True, 855770), (1, 128, 1, 1, 39, False, 111444), (1, 512, 4, 2, 267, True, 29219),
    (2, 256, 2, 1, 130, False, 169280), (1, 640, 6, 3, 516, True, 471007), (1, 512, 8, 1, 309, True, 295625),
    (1, 768, 4, 2, 576, True, 611097), (1, 384, 3, 3, 288, False, 591783), (2, 128, 8, 1, 52, False, 608064),
]


def test_model_error_sizes_support_the_gpu_bounds():
    scale = 1 / math.sqrt(128)
    worst = dict(store_only=0.0, worst=0.0, rms_lo=1.0, rms_hi=0.0, out=0.0, above_2e2=0, n=0)
    for (B, T, Hq, Hkv, W, gains, seed) in SWEEP:
        (q, k, v, dO), kw = inputs(B, T, Hq, Hkv, seed, gains)
        f = orc.fwd_dense(q, k, v, W, scale=scale, **kw)
        b = orc.bwd_dense(q, k, v, dO, W, scale=scale, **kw)
        m = em.model_fwd_bwd(q, k, v, dO, W, scale=scale, **kw)
        gmax = max(1.0, *(float(np.abs(g_).max()) for g_ in kw.values())) if gains else 1.0
        o = pm.out_err_bf16(m["o"], f["o"])
        worst["out"] = max(worst["out"], o["beyond_storage"] / gmax, o["raw_lt4"] / gmax)
        for n in ("dq", "dk", "dv"):
            ref = b[n]
            stored_only = pm.grad_err_bf16(em.bf16_round(ref), ref)
            assert stored_only["worst"] <= 1e-6           # the storage rounding is what `worst` takes off (fp32 step aside)
            worst["store_only"] = max(worst["store_only"], stored_only["raw"])
            g = pm.grad_err_bf16(m[n], ref)
            worst["worst"] = max(worst["worst"], g["worst"])
            worst["rms_lo"] = min(worst["rms_lo"], g["rms"]); worst["rms_hi"] = max(worst["rms_hi"], g["rms"])
            worst["above_2e2"] += g["worst"] > 2e-2
            worst["n"] += 1
    print(worst)
    # storing the exact gradient alone breaks "max|err| <= 2e-2 RMS"
    assert worst["store_only"] > 2e-2
    # bf16 operands: error sizes the GPU bounds are built on
    assert 2.4e-3 <= worst["rms_lo"] and worst["rms_hi"] <= 3.7e-3
    assert worst["rms_hi"] * pm.MODEL_RMS_FACTOR <= pm.GRAD_RMS_TOL
    assert 2e-2 < worst["worst"] <= 5e-2 and worst["above_2e2"] >= worst["n"] // 3
    assert worst["worst"] * 1.5 <= pm.GRAD_WORST_TOL <= worst["worst"] * 3.0   # head-room for a maximum, not a loose cap
    # the forward's output error keeps the stated 2e-2 (unit-scale outputs; gains scale it)
    assert worst["out"] <= pm.OUT_TOL_BF16


def test_model_sees_a_planted_mistake():
    """The relative-to-model criterion is not vacuous: an off-by-one in the window edge of the model's input (one key
    more in the softmax branch) moves the oracle-relative RMS error far beyond 1.2 x the model's own."""
    (q, k, v, dO), kw = inputs(1, 384, 2, 1, 77, False)
    scale = 1 / math.sqrt(128)
    ref = orc.bwd_dense(q, k, v, dO, 128, scale=scale)
    good = em.model_fwd_bwd(q, k, v, dO, 128, scale=scale)
    bad = orc.bwd_dense(q, k, v, dO, 129, scale=scale)      # exact arithmetic, wrong window
    for n in ("dq", "dk", "dv"):
        g, w = pm.grad_err_bf16(good[n], ref[n]), pm.grad_err_bf16(bad[n], ref[n])
        assert w["rms"] > pm.MODEL_RMS_FACTOR * g["rms"] + 1e-4, n
