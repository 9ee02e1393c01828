"""Seeded sweep of random shapes through the matrix-core kernels (bf16, D = 128): forward and backward against the
fp64 oracle, with the gradient criterion that needs no choice of seeds - the bf16 error model evaluated on the same
input (tests/bf16_error_model.py) - next to the absolute caps.  The sweep stops at its first failure.

Shapes: T = 128..895 (a third of them no multiple of the 128-row tile), 1..3 KV heads with group sizes 1..8, batch 1..3, any window from 8 keys to
beyond T (aligned and unaligned), gains on or off, gain gradients whenever there are gains."""
import math
import random

import numpy as np
import pytest
import torch

from oracle import rattn_oracle as orc
from paper_2506_15545_amd import binding as rb
from paper_2506_15545_amd import synth
import bf16_error_model as em
import parity_metrics as pm

pytestmark = pytest.mark.gpu

NCASES = 48


def np64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def draw_cases(n, seed=20250615):
    rng = random.Random(seed)
    cases = []
    for _ in range(n):
        T = 128 * rng.randint(1, 6)
        if rng.random() < 0.35:
            T += rng.randint(1, 127)       # a ragged length: the last, partial tile goes through the tail buffers
        G = rng.choice([1, 2, 3, 4, 6, 8])
        Hkv = rng.choice([1, 2, 3])
        B = rng.choice([1, 1, 2, 3])
        aligned = [64 * i for i in range(1, T // 64 + 1)] + [T, T + 64, 4 * T]
        W = rng.choice(aligned) if rng.random() < 0.3 else rng.randint(8, T + 3)
        cases.append((B, T, G * Hkv, Hkv, W, rng.random() < 0.5, rng.randint(0, 10 ** 6)))
    return cases


def test_random_shapes_against_oracle_and_error_model():
    scale = 1.0 / math.sqrt(128)
    for ci, (B, T, Hq, Hkv, W, gains, seed) in enumerate(draw_cases(NCASES)):
        print(f"random shape {ci}: B={B} T={T} Hq={Hq} Hkv={Hkv} W={W} gains={gains} seed={seed}", flush=True)
        x = synth.make_random_layer(B, T, Hq, Hkv, 128, "bf16", seed, with_dO=True, with_gains=gains)
        q, k, v, dO = (x[n].cuda() for n in ("q", "k", "v", "dO"))
        gs = x["gamma_swa"].cuda() if gains else None
        gr = x["gamma_rla"].cuda() if gains else None
        rb.rattn_profile_enable(True)
        o, saved = rb.rattn_fwd(q, k, v, W, gs, gr, softmax_scale=scale, save_for_bwd=True)
        dq, dk, dv, dgs, dgr = rb.rattn_bwd(q, k, v, saved, dO, W, gs, gr, softmax_scale=scale, want_dgamma=gains)
        torch.cuda.synchronize()
        names = [n for n, _ in rb.rattn_profile_records()]
        rb.rattn_profile_enable(False)
        assert "fwd_fused_kernel" in names and "bwd_dkv_kernel" in names
        kw = dict(gamma_swa=np64(x["gamma_swa"]), gamma_rla=np64(x["gamma_rla"])) if gains else {}
        args = [np64(x[n]) for n in ("q", "k", "v")]
        ref = orc.fwd_dense(*args, W, scale=scale, **kw)
        refb = orc.bwd_dense(*args, np64(x["dO"]), W, scale=scale, **kw)
        model = em.model_fwd_bwd(*args, np64(x["dO"]), W, scale=scale, **kw)
        gmax = max(1.0, float(x["gamma_swa"].abs().max()), float(x["gamma_rla"].abs().max())) if gains else 1.0
        pm.assert_out_bf16(np64(o), ref["o"], gmax, what=f"case {ci} o")
        for n, g_ in (("dq", dq), ("dk", dk), ("dv", dv)):
            pm.assert_grad_bf16(np64(g_), refb[n], f"case {ci} {n}", model[n])
        if gains:
            for n, g_ in (("dgamma_swa", dgs), ("dgamma_rla", dgr)):
                r = refb[n]
                if np.all(r == 0):
                    assert float(g_.abs().max()) <= 1e-6, n
                else:
                    e = float(np.max(np.abs(np64(g_) - r))) / math.sqrt(float(np.mean(r ** 2)))
                    assert e <= pm.GRAD_TOL_GENERAL, f"case {ci} {n}: {e}"
