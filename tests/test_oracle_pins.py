"""Pins for the fp64 oracle: things the paper and the mathematics fix, checked against
code that is not the oracle's own (library routines, autograd, finite differences,
closed forms, brute force).  CPU only."""
import itertools
import os
import numpy as np
import pytest
import scipy.special
import torch

from oracle import rattn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_layer(rng, B, T, Hq, Hkv, D, std=1.0):
    q = rng.standard_normal((B, T, Hq, D)) * std
    k = rng.standard_normal((B, T, Hkv, D)) * std
    v = rng.standard_normal((B, T, Hkv, D))
    return q, k, v


# ------------------------------------------------------------------ partition / lag (Fig. 1, Sec. 2.1, Eq. 4)
def test_fig1_worked_example():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "fig1_partition.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 2
    for W, t, res in rows:
        expect = [int(x) for x in res.split(",")]
        assert orc.residual_set_1based(int(t), int(W)) == expect
        assert len(orc.window_set_1based(int(t), int(W))) == int(W)


def test_partition_is_disjoint_cover_bruteforce():
    for W in range(0, 12):
        for t in range(1, 30):
            win = orc.window_set_1based(t, W); res = orc.residual_set_1based(t, W)
            assert sorted(win + res) == list(range(1, t + 1))
            assert len(win) <= max(W, 0)
            # paper's w = W-1: window holds at most w+1 tokens, state index is t-w-1
            if W >= 1:
                w = W - 1
                assert win == list(range(max(1, t - w), t + 1))
                assert res == list(range(1, t - w - 1 + 1))


def test_masks_match_index_sets():
    T = 23
    for W in (0, 1, 4, 7, 23, 40):
        win, res = orc._masks(np.arange(T), T, W)
        for t in range(T):
            assert [s + 1 for s in range(T) if win[t, s]] == orc.window_set_1based(t + 1, W)
            assert [s + 1 for s in range(T) if res[t, s]] == orc.residual_set_1based(t + 1, W)


# ------------------------------------------------------------------ phi
def test_phi_is_library_softmax():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7, 16)) * 3
    np.testing.assert_allclose(orc.phi(x), scipy.special.softmax(x, axis=-1), rtol=1e-14, atol=0)
    f = orc.phi(x)
    assert np.all(f > 0) and np.allclose(f.sum(-1), 1.0)


# ------------------------------------------------------------------ softmax branch vs library attention
def sdpa_f64(q, k, v, mask, scale):
    """torch's scaled_dot_product_attention in float64, one head: independent routine."""
    tq = torch.from_numpy(q)[None, None]; tk = torch.from_numpy(k)[None, None]; tv = torch.from_numpy(v)[None, None]
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(mask)[None, None],
                                                           scale=scale)
    return out[0, 0].numpy()


@pytest.mark.parametrize("W", [1, 3, 8, 33, 64])
def test_swa_branch_equals_library_banded_attention(W):
    rng = np.random.default_rng(1)
    B, T, Hq, Hkv, D = 2, 33, 4, 2, 8
    q, k, v = rand_layer(rng, B, T, Hq, Hkv, D)
    scale = 0.37
    out = orc.fwd_dense(q, k, v, W, scale=scale)
    t = np.arange(T)[:, None]; s = np.arange(T)[None, :]
    band = (s <= t) & (t - s < W)
    for b in range(B):
        for h in range(Hq):
            ref = sdpa_f64(q[b, :, h], k[b, :, h // 2], v[b, :, h // 2], band, scale)
            np.testing.assert_allclose(out["xs"][b, :, h], ref, rtol=1e-11, atol=1e-12)


def test_window_covering_sequence_is_causal_attention_and_no_residual():
    rng = np.random.default_rng(2)
    B, T, Hq, Hkv, D = 1, 40, 2, 1, 16
    q, k, v = rand_layer(rng, B, T, Hq, Hkv, D)
    eps = 1e-6
    for W in (T, T + 5):
        out = orc.fwd_dense(q, k, v, W, scale=0.25, eps=eps)
        assert np.all(out["xr"] == 0.0)
        for h in range(Hq):
            tq = torch.from_numpy(q[0, :, h])[None, None]; tk = torch.from_numpy(k[0, :, 0])[None, None]
            tv = torch.from_numpy(v[0, :, 0])[None, None]
            causal = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=0.25)[0, 0].numpy()
            np.testing.assert_allclose(out["xs"][0, :, h], causal, rtol=1e-11, atol=1e-12)
            # whole layer: o = RMS(causal attention), the empty branch contributes exactly 0
            ref_o = causal / np.sqrt((causal ** 2).mean(-1, keepdims=True) + eps)
            np.testing.assert_allclose(out["o"][0, :, h], ref_o, rtol=1e-11, atol=1e-12)


def test_softmax_branch_shift_invariance_and_lse():
    rng = np.random.default_rng(3)
    q, k, v = rand_layer(rng, 1, 20, 1, 1, 4)
    a = orc.fwd_dense(q, k, v, 5)
    # adding a constant vector c to every key shifts each logit row by q.c: softmax unchanged
    c = rng.standard_normal(4)
    b = orc.fwd_dense(q, k + c, v, 5)
    np.testing.assert_allclose(a["xs"], b["xs"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b["lse"] - a["lse"], (q[0, :, 0] @ c)[None, None, :], rtol=1e-10, atol=1e-10)


# ------------------------------------------------------------------ linear branch
@pytest.mark.parametrize("W,C", [(0, 4), (1, 4), (5, 4), (8, 8), (7, 16), (16, 5), (40, 8)])
def test_rla_recurrent_equals_masked_equals_chunkwise(W, C):
    rng = np.random.default_rng(4)
    q, k, v = rand_layer(rng, 2, 37, 4, 2, 8)
    rec = orc.rla_recurrent(q, k, v, W)
    dense = orc.fwd_dense(q, k, v, W)["xr"]
    chk = orc.rla_chunkwise(q, k, v, W, C)
    np.testing.assert_allclose(rec, dense, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(chk, dense, rtol=1e-11, atol=1e-13)
    if W > 0:
        assert np.all(dense[:, :W] == 0.0)       # queries t <= W (1-based) see an empty state, S_0 = 0


def test_window_zero_is_plain_linear_attention_eq1():
    rng = np.random.default_rng(5)
    q, k, v = rand_layer(rng, 1, 19, 1, 1, 6)
    ref = orc.linear_attention_eq1(q[0, :, 0], k[0, :, 0], v[0, :, 0])
    np.testing.assert_allclose(orc.fwd_dense(q, k, v, 0)["xr"][0, :, 0], ref, rtol=1e-11, atol=1e-13)
    # and Eq. 1 itself against a textbook double loop
    T = 19
    kf = scipy.special.softmax(k[0, :, 0], axis=-1); qf = scipy.special.softmax(q[0, :, 0], axis=-1)
    for t in (0, 7, 18):
        S = sum(np.outer(kf[s], v[0, s, 0]) for s in range(t + 1))
        np.testing.assert_allclose(ref[t], qf[t] @ S, rtol=1e-11, atol=1e-13)


def test_rla_shift_identity():
    # RLA(q,k,v;W)[t] = LA(q[W:], k[:T-W], v[:T-W])[t-W]
    rng = np.random.default_rng(6)
    T, W = 30, 9
    q, k, v = rand_layer(rng, 1, T, 1, 1, 5)
    xr = orc.fwd_dense(q, k, v, W)["xr"][0, :, 0]
    la = orc.linear_attention_eq1(q[0, W:, 0], k[0, :T - W, 0], v[0, :T - W, 0])
    np.testing.assert_allclose(xr[W:], la, rtol=1e-11, atol=1e-13)


def test_rla_equal_keys_closed_form():
    rng = np.random.default_rng(7)
    T, W, D = 25, 6, 8
    q, k, v = rand_layer(rng, 1, T, 1, 1, D)
    k[:] = k[0, 0, 0]
    kf = scipy.special.softmax(k[0, 0, 0])
    xr = orc.fwd_dense(q, k, v, W)["xr"][0, :, 0]
    csum = np.cumsum(v[0, :, 0], axis=0)
    for t in range(T):
        ref = np.zeros(D) if t - W < 0 else (scipy.special.softmax(q[0, t, 0]) @ kf) * csum[t - W]
        np.testing.assert_allclose(xr[t], ref, rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------ epilogue
def test_epilogue_properties():
    rng = np.random.default_rng(8)
    B, T, Hq, Hkv, D, W, eps = 1, 24, 2, 1, 8, 6, 1e-6
    q, k, v = rand_layer(rng, B, T, Hq, Hkv, D)
    out = orc.fwd_dense(q, k, v, W, eps=eps)
    # with unit gains each branch row has mean square m/(m+eps); empty rows are exactly 0
    for name in ("xs", "xr"):
        x = out[name]; m = (x ** 2).mean(-1)
        y = x / np.sqrt(m + eps)[..., None]
        np.testing.assert_allclose((y ** 2).mean(-1), m / (m + eps), rtol=1e-12)
    y_s = out["xs"] * out["rs"].transpose(0, 2, 1)[..., None]
    y_r = out["xr"] * out["rr"].transpose(0, 2, 1)[..., None]
    np.testing.assert_allclose(out["o"], y_s + y_r, rtol=1e-12, atol=1e-14)
    assert np.all(out["o"][:, :W] == y_s[:, :W])
    # both branches are linear in v, and RMS is scale-free up to eps: o(v) ~= o(7 v)
    out7 = orc.fwd_dense(q, k, 7.0 * v, W, eps=eps)
    np.testing.assert_allclose(out7["o"], out["o"], rtol=0, atol=1e-4)
    # gains are per head and per branch
    gs = rng.standard_normal((Hq, D)); gr = rng.standard_normal((Hq, D))
    outg = orc.fwd_dense(q, k, v, W, eps=eps, gamma_swa=gs, gamma_rla=gr)
    np.testing.assert_allclose(outg["o"], y_s * gs[None, None] + y_r * gr[None, None], rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ loops == dense, brute force
@pytest.mark.parametrize("W", [1, 2, 5, 16])
def test_loops_equal_dense(W):
    rng = np.random.default_rng(9)
    q, k, v = rand_layer(rng, 2, 13, 4, 2, 4)
    gs = rng.standard_normal((4, 4)); gr = rng.standard_normal((4, 4))
    a = orc.fwd_loops(q, k, v, W, scale=0.7, eps=1e-5, gamma_swa=gs, gamma_rla=gr)
    b = orc.fwd_dense(q, k, v, W, scale=0.7, eps=1e-5, gamma_swa=gs, gamma_rla=gr)
    for key in ("o", "xs", "xr"):
        np.testing.assert_allclose(a[key], b[key], rtol=1e-11, atol=1e-13)


def test_hand_expanded_three_tokens():
    # T=3, D=2, W=2, unit gains, scale 1: every sum written out by hand with math.exp
    import math
    q = np.array([[0.3, -0.2], [0.1, 0.5], [-0.4, 0.25]])
    k = np.array([[0.2, 0.1], [-0.3, 0.4], [0.05, -0.15]])
    v = np.array([[1.0, -2.0], [0.5, 0.25], [-1.5, 3.0]])
    eps = 1e-6
    out = orc.fwd_dense(q[None, :, None], k[None, :, None], v[None, :, None], 2, eps=eps)

    def sm2(x):
        e0, e1 = math.exp(x[0]), math.exp(x[1]); return [e0 / (e0 + e1), e1 / (e0 + e1)]

    def dot(a, b): return a[0] * b[0] + a[1] * b[1]
    # query 3 (index 2): window {2,3} (indices 1,2), residual {1} (index 0)
    e1 = math.exp(dot(q[2], k[1])); e2 = math.exp(dot(q[2], k[2]))
    xs = [(e1 * v[1][j] + e2 * v[2][j]) / (e1 + e2) for j in range(2)]
    c = dot(sm2(q[2]), sm2(k[0]))
    xr = [c * v[0][j] for j in range(2)]
    rs = 1 / math.sqrt((xs[0] ** 2 + xs[1] ** 2) / 2 + eps); rr = 1 / math.sqrt((xr[0] ** 2 + xr[1] ** 2) / 2 + eps)
    o = [xs[j] * rs + xr[j] * rr for j in range(2)]
    np.testing.assert_allclose(out["o"][0, 2, 0], o, rtol=1e-13)
    # query 1: window {1}, softmax weight 1, residual empty
    r0 = 1 / math.sqrt((v[0][0] ** 2 + v[0][1] ** 2) / 2 + eps)
    np.testing.assert_allclose(out["o"][0, 0, 0], [v[0][0] * r0, v[0][1] * r0], rtol=1e-13)


# ------------------------------------------------------------------ backward
def torch_layer(q, k, v, W, scale, eps, gs, gr):
    """Independent float64 autograd expression of the layer (torch ops, dense masks)."""
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]; G = Hq // Hkv
    kx = k.repeat_interleave(G, dim=2); vx = v.repeat_interleave(G, dim=2)
    t = torch.arange(T)[:, None]; s = torch.arange(T)[None, :]
    win = (s <= t) & (s > t - W); res = s <= t - W
    a = torch.einsum('bthd,bshd->bhts', q, kx) * scale
    a = a.masked_fill(~win, float('-inf'))
    xs = torch.einsum('bhts,bshd->bthd', torch.softmax(a, dim=-1), vx)
    c = torch.einsum('bthd,bshd->bhts', torch.softmax(q, -1), torch.softmax(kx, -1)) * res
    xr = torch.einsum('bhts,bshd->bthd', c, vx)
    n = lambda x, g: g * x * torch.rsqrt((x * x).mean(-1, keepdim=True) + eps)
    return n(xs, gs) + n(xr, gr)


@pytest.mark.parametrize("W,Hq,Hkv", [(1, 2, 2), (4, 4, 2), (7, 3, 1), (64, 2, 1)])
def test_backward_matches_autograd(W, Hq, Hkv):
    rng = np.random.default_rng(10)
    B, T, D = 2, 21, 8
    q, k, v = rand_layer(rng, B, T, Hq, Hkv, D)
    dO = rng.standard_normal(q.shape)
    gs = 1 + 0.3 * rng.standard_normal((Hq, D)); gr = 1 + 0.3 * rng.standard_normal((Hq, D))
    scale, eps = 0.4, 1e-5
    g = orc.bwd_dense(q, k, v, dO, W, scale=scale, eps=eps, gamma_swa=gs, gamma_rla=gr)
    tq, tk, tv, tgs, tgr = [torch.tensor(x, requires_grad=True) for x in (q, k, v, gs, gr)]
    out = torch_layer(tq, tk, tv, W, scale, eps, tgs, tgr)
    np.testing.assert_allclose(out.detach().numpy(),
                               orc.fwd_dense(q, k, v, W, scale=scale, eps=eps, gamma_swa=gs, gamma_rla=gr)["o"],
                               rtol=1e-10, atol=1e-12)
    out.backward(torch.from_numpy(dO))
    for name, tt in (("dq", tq), ("dk", tk), ("dv", tv), ("dgamma_swa", tgs), ("dgamma_rla", tgr)):
        np.testing.assert_allclose(g[name], tt.grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=name)


def test_backward_matches_finite_differences():
    rng = np.random.default_rng(11)
    B, T, Hq, Hkv, D, W = 1, 9, 2, 1, 4, 3
    q, k, v = rand_layer(rng, B, T, Hq, Hkv, D)
    dO = rng.standard_normal(q.shape)
    scale, eps = 0.9, 1e-3
    g = orc.bwd_dense(q, k, v, dO, W, scale=scale, eps=eps)
    f = lambda q_, k_, v_: np.sum(orc.fwd_loops(q_, k_, v_, W, scale=scale, eps=eps)["o"] * dO)
    h = 1e-6
    for name, arr, idx in (("dq", q, 0), ("dk", k, 1), ("dv", v, 2)):
        num = np.zeros_like(arr)
        for i in itertools.product(*[range(n) for n in arr.shape]):
            args = [q.copy(), k.copy(), v.copy()]
            args[idx][i] += h; fp = f(*args)
            args[idx][i] -= 2 * h; fm = f(*args)
            num[i] = (fp - fm) / (2 * h)
        np.testing.assert_allclose(g[name], num, rtol=2e-6, atol=2e-8, err_msg=name)


def test_backward_row_restriction_is_additive():
    rng = np.random.default_rng(12)
    q, k, v = rand_layer(rng, 1, 17, 2, 1, 4)
    dO = rng.standard_normal(q.shape)
    full = orc.bwd_dense(q, k, v, dO, 5)
    a = orc.bwd_dense(q, k, v, dO, 5, rows=np.arange(0, 8))
    b = orc.bwd_dense(q, k, v, dO, 5, rows=np.arange(8, 17))
    for name in ("dq", "dk", "dv", "dgamma_swa", "dgamma_rla"):
        np.testing.assert_allclose(a[name] + b[name], full[name], rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------ decode
@pytest.mark.parametrize("W,T", [(4, 15), (1, 6), (6, 6), (9, 5)])
def test_decode_chain_reproduces_forward(W, T):
    rng = np.random.default_rng(13)
    N, Hq, Hkv, D = 2, 4, 2, 6
    q, k, v = rand_layer(rng, N, T, Hq, Hkv, D)
    gs = 1 + 0.2 * rng.standard_normal((Hq, D)); gr = 1 + 0.2 * rng.standard_normal((Hq, D))
    ref = orc.fwd_dense(q, k, v, W, scale=0.5, eps=1e-6, gamma_swa=gs, gamma_rla=gr)["o"]
    kr = np.zeros((N, Hkv, W, D)); vr = np.zeros((N, Hkv, W, D)); S = np.zeros((N, Hkv, D, D))
    for t in range(T):
        o, kr, vr, S = orc.decode_step(q[:, t], k[:, t], v[:, t], np.full(N, t), kr, vr, S, W,
                                       scale=0.5, eps=1e-6, gamma_swa=gs, gamma_rla=gr)
        np.testing.assert_allclose(o, ref[:, t], rtol=1e-10, atol=1e-12)
        # slot convention: key t sits in slot t % W
        np.testing.assert_array_equal(kr[:, :, t % W], k[:, t])
    # the state ends as the sum over keys 0..T-1-W
    kf = scipy.special.softmax(k, axis=-1)
    Sref = np.einsum('nsgf,nsgd->ngfd', kf[:, :max(T - W, 0)], v[:, :max(T - W, 0)])
    np.testing.assert_allclose(S, Sref, rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------ closed forms printed in the text
def test_text_closed_forms():
    # Sec. 1: 12B model (40 layers, 1 global per 4), 4K context, window 4K -> 1K: ~56 %
    assert abs(orc.kv_cache_saving(40, 4, 4096, 4096, 1024) - 0.5625) < 1e-12
    # Sec. 2.2 footnote: a 128 x 128 state costs as much as a 64-token window
    assert orc.state_equivalent_window(128, 128) == 64


def test_state_equivalent_window_counts_cache_elements():
    """Sec. 2.2: the state is as large as the key/value cache of that many tokens.  Pinned by counting array elements:
    the first window length whose cache of keys and values (one row of d each per token) holds as many numbers as
    the d' x d state."""
    for d_feat, d in ((128, 128), (256, 128), (64, 64), (128, 64)):
        state_numbers = np.zeros((d_feat, d)).size
        n = next(n for n in range(1, 10000) if np.zeros((n, 2, d)).size >= state_numbers)
        assert orc.state_equivalent_window(d_feat, d) == n, (d_feat, d)


def test_decode_step_time_hand_evaluated_cases():
    """Sec. 4.4 step-time model, two cases worked by hand (cache term + the larger of the compute and weight terms).
    Hardware: 2e12 B/s, 1e15 FLOP/s; model: 3e9 parameters in 6e9 bytes; cache 1e9 bytes per sequence.
      batch 4096: cache 4096e9/2e12 = 2.048 s; compute 2*4096*3e9/1e15 = 0.024576 s > weights 6e9/2e12 = 0.003 s
                  -> 2.072576 s (compute-bound)
      batch 1:    cache 1e9/2e12 = 0.0005 s; compute 2*3e9/1e15 = 0.000006 s < weights 0.003 s -> 0.0035 s (weight-bound)"""
    assert abs(orc.decode_step_time(4096, 1e9, 3e9, 6e9, 2e12, 1e15) - 2.072576) < 1e-12
    assert abs(orc.decode_step_time(1, 1e9, 3e9, 6e9, 2e12, 1e15) - 0.0035) < 1e-15
    # a faster matrix unit moves only the compute-bound case; a wider memory system moves both
    assert abs(orc.decode_step_time(4096, 1e9, 3e9, 6e9, 2e12, 2e15) - (2.048 + 0.012288)) < 1e-12
    assert abs(orc.decode_step_time(1, 1e9, 3e9, 6e9, 2e12, 2e15) - 0.0035) < 1e-15
    assert abs(orc.decode_step_time(1, 1e9, 3e9, 6e9, 4e12, 1e15) - 0.00175) < 1e-15


# ------------------------------------------------------------------------------ prefill -> decode hand-over
@pytest.mark.parametrize("T,W", [(3, 8), (8, 8), (9, 8), (21, 4), (16, 1)])
def test_prefill_export_equals_decode_chain(T, W):
    """The exported rings/state are what T decode steps from empty rings and a zero state leave behind, and a
    decode step on top of them reproduces row T of the full forward pass over T+1 tokens."""
    rng = np.random.default_rng(70 + T + W)
    B, Hq, Hkv, D = 2, 4, 2, 4
    q = rng.standard_normal((B, T + 1, Hq, D)); k = rng.standard_normal((B, T + 1, Hkv, D))
    v = rng.standard_normal((B, T + 1, Hkv, D))
    kr = np.zeros((B, Hkv, W, D)); vr = np.zeros((B, Hkv, W, D)); S = np.zeros((B, Hkv, D, D))
    for t in range(T):
        _, kr, vr, S = orc.decode_step(q[:, t], k[:, t], v[:, t], [t] * B, kr, vr, S, W, scale=0.5)
    kr2, vr2, S2 = orc.prefill_export(k[:, :T], v[:, :T], W)
    assert np.array_equal(kr, kr2) and np.array_equal(vr, vr2)
    assert np.allclose(S, S2, rtol=1e-12, atol=1e-12)
    o, _, _, _ = orc.decode_step(q[:, T], k[:, T], v[:, T], [T] * B, kr2, vr2, S2, W, scale=0.5)
    ref = orc.fwd_dense(q, k, v, W, scale=0.5)["o"][:, T]
    assert np.allclose(o, ref, rtol=1e-9, atol=1e-9)


def test_prefill_export_state_is_cumulative_outer_products():
    rng = np.random.default_rng(5)
    k = rng.standard_normal((1, 12, 1, 3)); v = rng.standard_normal((1, 12, 1, 3))
    _, _, S = orc.prefill_export(k, v, 5)
    f = np.exp(k[0, :7, 0]); f /= f.sum(axis=1, keepdims=True)      # softmax rows of the 7 out-of-window keys
    assert np.allclose(S[0, 0], f.T @ v[0, :7, 0], rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------------------ feature-map variants (Sec. 4.5 ablation)
TORCH_PHI = {"softmax": lambda x: torch.softmax(x, -1), "relu": torch.relu, "identity": lambda x: x}
NUMPY_PHI = {"softmax": lambda x: scipy.special.softmax(x, axis=-1), "relu": lambda x: np.where(x > 0, x, 0.0),
             "identity": lambda x: x}
VARIANTS = ("relu", "identity")


def test_variant_feature_maps_on_printed_values():
    x = np.array([[-1.5, 0.0, 2.0, -0.0, 3.25]])
    assert np.array_equal(orc.phi(x, "relu"), [[0.0, 0.0, 2.0, 0.0, 3.25]])
    assert np.array_equal(orc.phi(x, "identity"), x)
    assert orc.phi(x, "identity") is not x
    with pytest.raises(ValueError):
        orc.phi(x, "elu")
    # gradients through phi against autograd, every map
    rng = np.random.default_rng(40)
    xx = rng.standard_normal((6, 9)); df = rng.standard_normal((6, 9))
    for name, fn in TORCH_PHI.items():
        t = torch.tensor(xx, requires_grad=True)
        (fn(t) * torch.from_numpy(df)).sum().backward()
        np.testing.assert_allclose(orc.phi_bwd(xx, orc.phi(xx, name), df, name), t.grad.numpy(), rtol=1e-12, atol=1e-14,
                                   err_msg=name)


@pytest.mark.parametrize("fm", VARIANTS)
@pytest.mark.parametrize("W,C", [(0, 4), (3, 4), (8, 8), (7, 16), (40, 8)])
def test_variant_linear_branch_forms_agree_and_match_cumulative_sums(fm, W, C):
    """Recurrent (Eq. 4), masked and chunkwise (Eqs. 2-3) forms agree for the ablation's maps, and all equal the
    textbook expression phi(q_t) . cumsum_s(phi(k_s)^T v_s)[t - W] written with library cumsum/einsum."""
    rng = np.random.default_rng(41)
    q, k, v = rand_layer(rng, 2, 37, 4, 2, 8)
    rec = orc.rla_recurrent(q, k, v, W, feature_map=fm)
    dense = orc.fwd_dense(q, k, v, W, feature_map=fm)["xr"]
    chk = orc.rla_chunkwise(q, k, v, W, C, feature_map=fm)
    loops = orc.fwd_loops(q[:1, :12], k[:1, :12], v[:1, :12], W, feature_map=fm)["xr"]
    np.testing.assert_allclose(rec, dense, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(chk, dense, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(loops, dense[:1, :12], rtol=1e-11, atol=1e-12)
    f = NUMPY_PHI[fm]
    S = np.cumsum(np.einsum('btgf,btgd->btgfd', f(k), v), axis=1)            # S[b, s] = sum over keys <= s
    G = q.shape[2] // k.shape[2]
    for t in (0, W, W + 1, 20, 36):
        if t >= 37:
            continue
        for h in range(q.shape[2]):
            ref = np.zeros((2, 8)) if t - W < 0 else np.einsum('bf,bfd->bd', f(q[:, t, h]), S[:, t - W, h // G])
            np.testing.assert_allclose(dense[:, t, h], ref, rtol=1e-11, atol=1e-12)


def test_variant_special_cases():
    rng = np.random.default_rng(42)
    q, k, v = rand_layer(rng, 1, 20, 2, 1, 6)
    # positive q and k: ReLU is the identity map
    a = orc.fwd_dense(np.abs(q), np.abs(k), v, 5, feature_map="relu")
    b = orc.fwd_dense(np.abs(q), np.abs(k), v, 5, feature_map="identity")
    np.testing.assert_allclose(a["o"], b["o"], rtol=1e-13, atol=0)
    # keys with no positive feature contribute nothing under ReLU: the linear branch vanishes, and o = RMS_s(x^s)
    c = orc.fwd_dense(q, -np.abs(k), v, 5, feature_map="relu")
    assert np.all(c["xr"] == 0.0)
    np.testing.assert_allclose(c["o"], orc.rms(c["xs"], 1.0, 1e-6)[0], rtol=1e-13, atol=0)
    # identity: the branch is bilinear in (q, k) - softmax is not - and the softmax branch does not depend on the map
    d1 = orc.fwd_dense(q, k, v, 5, feature_map="identity")
    d2 = orc.fwd_dense(2.0 * q, k, v, 5, feature_map="identity")
    d3 = orc.fwd_dense(q, -3.0 * k, v, 5, feature_map="identity")
    np.testing.assert_allclose(d2["xr"], 2.0 * d1["xr"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(d3["xr"], -3.0 * d1["xr"], rtol=1e-12, atol=1e-13)
    s0 = orc.fwd_dense(q, k, v, 5)
    assert np.array_equal(s0["xs"], d1["xs"]) and np.array_equal(s0["lse"], d1["lse"])
    assert not np.allclose(s0["xr"], d1["xr"])


def torch_layer_fm(q, k, v, W, scale, eps, gs, gr, fm):
    """torch_layer with the feature map of the linear branch exchanged."""
    B, T, Hq, D = q.shape
    G = Hq // k.shape[2]
    kx = k.repeat_interleave(G, dim=2); vx = v.repeat_interleave(G, dim=2)
    t = torch.arange(T)[:, None]; s = torch.arange(T)[None, :]
    win = (s <= t) & (s > t - W); res = s <= t - W
    a = (torch.einsum('bthd,bshd->bhts', q, kx) * scale).masked_fill(~win, float('-inf'))
    xs = torch.einsum('bhts,bshd->bthd', torch.softmax(a, dim=-1), vx)
    c = torch.einsum('bthd,bshd->bhts', TORCH_PHI[fm](q), TORCH_PHI[fm](kx)) * res
    xr = torch.einsum('bhts,bshd->bthd', c, vx)
    n = lambda x, g: g * x * torch.rsqrt((x * x).mean(-1, keepdim=True) + eps)
    return n(xs, gs) + n(xr, gr)


@pytest.mark.parametrize("fm", VARIANTS)
@pytest.mark.parametrize("W,Hq,Hkv", [(1, 2, 2), (4, 4, 2), (7, 3, 1)])
def test_variant_backward_matches_autograd(fm, W, Hq, Hkv):
    rng = np.random.default_rng(43)
    B, T, D = 2, 21, 8
    q, k, v = rand_layer(rng, B, T, Hq, Hkv, D)
    dO = rng.standard_normal(q.shape)
    gs = 1 + 0.3 * rng.standard_normal((Hq, D)); gr = 1 + 0.3 * rng.standard_normal((Hq, D))
    scale, eps = 0.4, 1e-5
    g = orc.bwd_dense(q, k, v, dO, W, scale=scale, eps=eps, gamma_swa=gs, gamma_rla=gr, feature_map=fm)
    tq, tk, tv, tgs, tgr = [torch.tensor(x, requires_grad=True) for x in (q, k, v, gs, gr)]
    out = torch_layer_fm(tq, tk, tv, W, scale, eps, tgs, tgr, fm)
    ref = orc.fwd_dense(q, k, v, W, scale=scale, eps=eps, gamma_swa=gs, gamma_rla=gr, feature_map=fm)["o"]
    np.testing.assert_allclose(out.detach().numpy(), ref, rtol=1e-10, atol=1e-12)
    out.backward(torch.from_numpy(dO))
    for name, tt in (("dq", tq), ("dk", tk), ("dv", tv), ("dgamma_swa", tgs), ("dgamma_rla", tgr)):
        np.testing.assert_allclose(g[name], tt.grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=name)


@pytest.mark.parametrize("fm", VARIANTS)
def test_variant_decode_chain_and_export(fm):
    rng = np.random.default_rng(44)
    N, T, Hq, Hkv, D, W = 2, 15, 4, 2, 6, 4
    q, k, v = rand_layer(rng, N, T, Hq, Hkv, D)
    ref = orc.fwd_dense(q, k, v, W, scale=0.5, feature_map=fm)["o"]
    kr = np.zeros((N, Hkv, W, D)); vr = np.zeros((N, Hkv, W, D)); S = np.zeros((N, Hkv, D, D))
    for t in range(T):
        if t == 11:
            kr2, vr2, S2 = orc.prefill_export(k[:, :t], v[:, :t], W, feature_map=fm)
            assert np.array_equal(kr, kr2) and np.array_equal(vr, vr2)
            np.testing.assert_allclose(S, S2, rtol=1e-12, atol=1e-13)
        o, kr, vr, S = orc.decode_step(q[:, t], k[:, t], v[:, t], np.full(N, t), kr, vr, S, W, scale=0.5,
                                       feature_map=fm)
        np.testing.assert_allclose(o, ref[:, t], rtol=1e-10, atol=1e-12)
    Sref = np.einsum('nsgf,nsgd->ngfd', NUMPY_PHI[fm](k[:, :T - W]), v[:, :T - W])
    np.testing.assert_allclose(S, Sref, rtol=1e-11, atol=1e-13)
