"""GPU parity for the ablation's feature maps of the linear branch (Sec. 4.5: ReLU and identity instead of the
softmax map): forward, backward, decode, prefill export and chunked prefill through the C ABI against the fp64
oracle, to the same bars as the softmax map (max-abs 1e-4 fp32 / 2e-2 bf16 on unit-scale outputs; gradients relative
to the RMS of the oracle gradient; on the matrix-core kernels, which take the ReLU map as well, the two-part
gradient bound of those kernels)."""
import math
import numpy as np
import pytest
import torch

from oracle import rattn_oracle as orc
from paper_2506_15545_amd import binding as rb
from paper_2506_15545_amd import synth
import bf16_error_model as em
import parity_metrics as pm

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
MAPS = ("relu", "identity")


def np64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def out_err(got, ref, dtype):
    e = np.abs(np64(got) - ref)
    if dtype == "bf16":
        e = np.maximum(e - pm.half_ulp_bf16(ref), 0.0)   # rounding of the stored value itself
    return float(e.max())


def grad_err(got, ref, dtype):
    return out_err(got, ref, dtype) / (math.sqrt(float(np.mean(ref ** 2))) + 1e-30)


def kernels_of(fn):
    rb.rattn_profile_enable(True)
    out = fn()
    torch.cuda.synchronize()
    names = [n for n, _ in rb.rattn_profile_records()]
    rb.rattn_profile_enable(False)
    return out, names


def layer_case(fm, B, T, Hq, Hkv, D, W, dtype, seed, chunk=0, backward=True, mfma=False):
    x = synth.make_random_layer(B, T, Hq, Hkv, D, dtype, seed, with_dO=True, with_gains=True)
    scale = 1.0 / math.sqrt(D)
    print(f"feature map {fm}: B={B} T={T} Hq={Hq} Hkv={Hkv} D={D} W={W} {dtype} chunk={chunk} seed={seed}", flush=True)
    q, k, v, dO, gs, gr = [x[n].cuda() for n in ("q", "k", "v", "dO", "gamma_swa", "gamma_rla")]
    kw = dict(gamma_swa=np64(x["gamma_swa"]), gamma_rla=np64(x["gamma_rla"]), scale=scale, feature_map=fm)
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, **kw)
    gmax = max(float(gs.abs().max()), float(gr.abs().max()), 1.0)
    if mfma and fm == "identity":
        # the identity map runs on the matrix cores only where nothing is kept for a backward pass (its backward is
        # not accurate enough with bf16 operands): the forward alone here, the training step below on the general kernels
        o_inf, names = kernels_of(lambda: rb.rattn_fwd(q, k, v, W, gs, gr, chunk=chunk, softmax_scale=scale,
                                                       feature_map=fm))
        assert "fwd_fused_kernel" in names and "gen_fwd_kernel" not in names
        pm.assert_out_bf16(np64(o_inf), ref["o"], gmax, what="identity, forward only")
        mfma = False
    (o, saved), names = kernels_of(lambda: rb.rattn_fwd(q, k, v, W, gs, gr, chunk=chunk, softmax_scale=scale,
                                                        save_for_bwd=True, feature_map=fm))
    assert ("fwd_fused_kernel" in names) == mfma and ("gen_fwd_kernel" in names) == (not mfma)
    if dtype == "bf16":
        pm.assert_out_bf16(np64(o), ref["o"], gmax)
    else:
        assert out_err(o, ref["o"], dtype) <= TOL[dtype] * gmax
    if not backward:
        return
    (dq, dk, dv, dgs, dgr), names = kernels_of(lambda: rb.rattn_bwd(q, k, v, saved, dO, W, gs, gr, chunk=chunk,
                                                                    softmax_scale=scale, feature_map=fm))
    assert ("bwd_dkv_kernel" in names) == mfma and ("gen_bwd_dkv_kernel" in names) == (not mfma)
    g = orc.bwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), np64(x["dO"]), W, **kw)
    model = None
    if mfma:  # the bf16 error model on the same input (same feature map)
        model = em.model_fwd_bwd(np64(x["q"]), np64(x["k"]), np64(x["v"]), np64(x["dO"]), W, scale=scale,
                                 gamma_swa=kw["gamma_swa"], gamma_rla=kw["gamma_rla"], feature_map=fm)
    for name, got in (("dq", dq), ("dk", dk), ("dv", dv), ("dgamma_swa", dgs), ("dgamma_rla", dgr)):
        if mfma and not name.startswith("dgamma"):
            pm.assert_grad_bf16(np64(got), g[name], f"{fm} {name}", model[name])
            continue
        e = grad_err(got, g[name], "f32" if name.startswith("dgamma") else dtype)
        assert e <= TOL[dtype], f"{name}: {e}"


@pytest.mark.parametrize("fm", MAPS)
@pytest.mark.parametrize("B,T,Hq,Hkv,D,W,chunk", [
    (2, 77, 4, 2, 64, 5, 0),         # ragged length, small window, two heads per group
    (1, 130, 3, 1, 128, 33, 16),     # three heads per group, odd window, short chunks
    (1, 150, 2, 1, 64, 1, 7),        # window of one key
    (1, 260, 2, 2, 128, 70, 100),    # intra-chunk part longer than one pass of the wave
    (1, 96, 2, 2, 64, 96, 0),        # window = T: no linear branch, the map must not matter
])
def test_layer_f32(fm, B, T, Hq, Hkv, D, W, chunk):
    layer_case(fm, B, T, Hq, Hkv, D, W, "f32", 900 + T, chunk)


@pytest.mark.parametrize("fm", MAPS)
@pytest.mark.parametrize("B,T,Hq,Hkv,D,W", [(1, 256, 4, 2, 128, 64), (2, 333, 2, 1, 64, 20), (1, 1100, 2, 1, 128, 100),
                                              (2, 100, 2, 1, 64, 20), (1, 90, 2, 2, 128, 30)])
def test_layer_bf16(fm, B, T, Hq, Hkv, D, W):
    # from one 128-row tile on, the matrix-core kernels (ragged lengths, head size 64 included); shorter sequences on
    # the general kernels (identity map: matrix cores for forward-only calls)
    layer_case(fm, B, T, Hq, Hkv, D, W, "bf16", 950 + T, mfma=(T >= 128))


@pytest.mark.parametrize("B,T,Hq,Hkv,W", [
    (1, 128, 2, 1, 64), (2, 512, 4, 2, 128), (1, 1024, 3, 1, 192), (1, 768, 2, 1, 512), (1, 384, 2, 2, 384),
    (1, 1024, 2, 1, 513), (1, 384, 3, 1, 100), (2, 256, 2, 2, 10), (1, 896, 2, 1, 320), (1, 256, 2, 1, 250),
])
@pytest.mark.parametrize("fm", MAPS)
def test_variant_maps_on_the_matrix_core_kernels(fm, B, T, Hq, Hkv, W):
    """Both state alignments, windows that are no tile multiples, a half-full last key tile, causal degenerate case."""
    layer_case(fm, B, T, Hq, Hkv, 128, W, "bf16", 1900 + T + W, mfma=True)


def test_kernel_selection_and_maps_differ():
    x = synth.make_random_layer(1, 256, 2, 1, 128, "bf16", 960)
    q, k, v = x["q"].cuda(), x["k"].cuda(), x["v"].cuda()
    outs = {}
    for fm in ("softmax",) + MAPS:
        outs[fm], names = kernels_of(lambda: rb.rattn_fwd(q, k, v, 64, softmax_scale=0.09, feature_map=fm))
        assert "fwd_fused_kernel" in names and "gen_fwd_kernel" not in names   # all three maps on the matrix cores
    # rows inside the first window have no linear branch: the map cannot matter there; later rows differ
    assert torch.equal(outs["relu"][:, :64], outs["softmax"][:, :64])
    assert float((outs["relu"][:, :64].float() - outs["identity"][:, :64].float()).abs().max()) <= 2e-2
    assert float((outs["relu"][:, 64:].float() - outs["identity"][:, 64:].float()).abs().max()) > 0.1
    assert float((outs["softmax"][:, 64:].float() - outs["identity"][:, 64:].float()).abs().max()) > 0.1


@pytest.mark.parametrize("fm", MAPS)
@pytest.mark.parametrize("dtype,D,Hq,Hkv,W,T", [("f32", 64, 4, 2, 8, 30), ("bf16", 128, 4, 1, 16, 40),
                                                 ("bf16", 128, 8, 1, 8, 20), ("f32", 128, 3, 1, 5, 12)])
def test_decode_chain_reproduces_forward(fm, dtype, D, Hq, Hkv, W, T):
    """T decode steps from empty rings and a zero state give the rows of the forward (oracle), and the state ends
    as the oracle's export of the whole sequence."""
    N = 2
    x = synth.make_random_layer(N, T, Hq, Hkv, D, dtype, 970 + T, with_gains=True)
    scale = 1.0 / math.sqrt(D)
    gs, gr = x["gamma_swa"], x["gamma_rla"]
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, scale=scale, gamma_swa=np64(gs),
                        gamma_rla=np64(gr), feature_map=fm)["o"]
    q, k, v = x["q"].cuda(), x["k"].cuda(), x["v"].cuda()
    kr = torch.zeros(N, Hkv, W, D, dtype=q.dtype, device="cuda"); vr = torch.zeros_like(kr)
    S = torch.zeros(N, Hkv, D, D, dtype=torch.float32, device="cuda")
    gmax = max(float(gs.abs().max()), float(gr.abs().max()), 1.0)
    for t in range(T):
        pos = torch.full((N,), t, dtype=torch.int32, device="cuda")
        o = rb.rattn_decode_step(q[:, t].contiguous(), k[:, t].contiguous(), v[:, t].contiguous(), pos, kr, vr, S,
                                 gs.cuda(), gr.cuda(), softmax_scale=scale, feature_map=fm)
        assert out_err(o, ref[:, t], dtype) <= TOL[dtype] * gmax, t
    _, _, S_ref = orc.prefill_export(np64(x["k"]), np64(x["v"]), W, feature_map=fm)
    assert float(np.max(np.abs(np64(S) - S_ref))) <= 2e-5 * max(1.0, float(np.abs(S_ref).max()))


@pytest.mark.parametrize("fm", MAPS)
@pytest.mark.parametrize("dtype,T,D,W", [("f32", 77, 64, 10), ("bf16", 1000, 128, 200)])
def test_prefill_export_then_decode(fm, dtype, T, D, W):
    B, Hq, Hkv = 2, 4, 2
    x = synth.make_random_layer(B, T + 1, Hq, Hkv, D, dtype, 980 + T)
    scale = 1.0 / math.sqrt(D)
    kr_ref, vr_ref, S_ref = orc.prefill_export(np64(x["k"][:, :T]), np64(x["v"][:, :T]), W, feature_map=fm)
    q, k, v = x["q"].cuda(), x["k"].cuda(), x["v"].cuda()
    kr, vr, S = rb.rattn_prefill_export(k[:, :T].contiguous(), v[:, :T].contiguous(), W, feature_map=fm)
    assert np.array_equal(np64(kr), kr_ref) and np.array_equal(np64(vr), vr_ref)
    assert float(np.max(np.abs(np64(S) - S_ref))) <= 2e-5 * max(1.0, float(np.abs(S_ref).max()))
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, scale=scale, rows=np.array([T]),
                        feature_map=fm)["o"][:, T]
    pos = torch.full((B,), T, dtype=torch.int32, device="cuda")
    o = rb.rattn_decode_step(q[:, T].contiguous(), k[:, T].contiguous(), v[:, T].contiguous(), pos, kr, vr, S,
                             softmax_scale=scale, feature_map=fm)
    assert out_err(o, ref, dtype) <= TOL[dtype]


@pytest.mark.parametrize("fm", MAPS)
@pytest.mark.parametrize("dtype,D,Hq,Hkv,W,chunks", [
    ("f32", 64, 4, 2, 8, [5, 3, 9, 1, 12]),
    ("bf16", 128, 4, 2, 128, [128, 256, 128]),     # whole tiles: the softmax map would take the matrix-core route
    ("bf16", 128, 2, 1, 100, [1100, 500]),
])
def test_chunked_prefill_reproduces_forward(fm, dtype, D, Hq, Hkv, W, chunks):
    B, T = 2, sum(chunks)
    x = synth.make_random_layer(B, T, Hq, Hkv, D, dtype, 990 + T + W, with_gains=True)
    scale = 1.0 / math.sqrt(D)
    gs, gr = x["gamma_swa"], x["gamma_rla"]
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, scale=scale, gamma_swa=np64(gs),
                        gamma_rla=np64(gr), feature_map=fm)["o"]
    kr_ref, vr_ref, S_ref = orc.prefill_export(np64(x["k"]), np64(x["v"]), W, feature_map=fm)
    q, k, v = x["q"].cuda(), x["k"].cuda(), x["v"].cuda()
    kr = torch.zeros(B, Hkv, W, D, dtype=q.dtype, device="cuda"); vr = torch.zeros_like(kr)
    S = torch.full((B, Hkv, D, D), float("nan"), dtype=torch.float32, device="cuda")
    gmax = max(float(gs.abs().max()), float(gr.abs().max()), 1.0)
    pos0 = 0
    for n in chunks:
        print(f"chunked prefill ({fm}) {dtype} D={D} W={W}: tokens {pos0}..{pos0 + n - 1}", flush=True)
        sl = slice(pos0, pos0 + n)
        o = rb.rattn_prefill_chunk(q[:, sl].contiguous(), k[:, sl].contiguous(), v[:, sl].contiguous(), W, pos0, kr, vr,
                                   S, gs.cuda(), gr.cuda(), softmax_scale=scale, feature_map=fm)
        torch.cuda.synchronize()
        assert out_err(o, ref[:, sl], dtype) <= TOL[dtype] * gmax, pos0
        pos0 += n
    assert np.array_equal(np64(kr), kr_ref) and np.array_equal(np64(vr), vr_ref)
    assert float(np.max(np.abs(np64(S) - S_ref))) <= 2e-5 * max(1.0, float(np.abs(S_ref).max()))
