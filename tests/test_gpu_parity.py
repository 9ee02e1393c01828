"""GPU parity: librattn (through the C ABI binding) against the fp64 oracle, element by element,
on seeded synthetic inputs.  Tolerances: max-abs 1e-4 for fp32 tensors and 2e-2 for bf16 tensors,
relative to unit-scale outputs (outputs are RMS-normalised; gradients are divided by the RMS of
the oracle gradient)."""
import math
import numpy as np
import pytest
import torch

from oracle import rattn_oracle as orc
from paper_2506_15545_amd import binding as rb
from paper_2506_15545_amd import synth
import parity_metrics as pm

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def np64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def dev(t):
    return None if t is None else t.cuda()


def maxerr(got, ref):
    return float(np.max(np.abs(np64(got) - ref)))


def rel_rms_err(got, ref, dtype="f32"):
    """max |got-ref| / RMS(ref).  Gradients are heavy-tailed (max ~ 10 RMS), so for bf16 tensors the
    unavoidable rounding of the stored value itself (half a bf16 ulp of the exact value) is taken off
    before dividing: the exact gradient rounded to bf16 scores 0.  The raw figure is printed."""
    rms = math.sqrt(float(np.mean(ref ** 2))) + 1e-30
    err = np.abs(np64(got) - ref)
    if dtype == "bf16":
        print(f"    raw max|err|/RMS {float(err.max()) / rms:.4f}", flush=True)
        err = np.maximum(err - pm.half_ulp_bf16(ref), 0.0)
    return float(np.max(err)) / rms


def run_fwd_case(B, T, Hq, Hkv, D, W, dtype, seed, chunk=0, scale=None, gains=False, std=1.0, eps=1e-6):
    x = synth.make_random_layer(B, T, Hq, Hkv, D, dtype, seed, std=std, with_gains=gains)
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    gs, gr = x.get("gamma_swa"), x.get("gamma_rla")
    print(f"fwd case B={B} T={T} Hq={Hq} Hkv={Hkv} D={D} W={W} {dtype} chunk={chunk} seed={seed}", flush=True)
    o = rb.rattn_fwd(dev(x["q"]), dev(x["k"]), dev(x["v"]), W, dev(gs), dev(gr), chunk=chunk, softmax_scale=scale,
                     rms_eps=eps)
    torch.cuda.synchronize()
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, scale=scale, eps=eps,
                        gamma_swa=None if gs is None else np64(gs), gamma_rla=None if gr is None else np64(gr))
    # gains scale the output; keep the bar relative to unit-scale rows
    gmax = 1.0 if gs is None else max(float(gs.abs().max()), float(gr.abs().max()), 1.0)
    err = maxerr(o, ref["o"])
    assert err <= TOL[dtype] * gmax, f"max abs err {err}"
    return err


def test_config1_tiny_f32_against_explicit_loops():
    cfg = synth.CONFIGS["tiny_f32"]
    q, k, v = synth.make_layer_inputs(cfg)
    o = rb.rattn_fwd(q.cuda(), k.cuda(), v.cuda(), cfg.W, chunk=cfg.chunk, softmax_scale=cfg.scale)
    ref = orc.fwd_loops(np64(q), np64(k), np64(v), cfg.W, scale=cfg.scale)
    assert maxerr(o, ref["o"]) <= 1e-4


@pytest.mark.parametrize("B,T,Hq,Hkv,D,W,chunk", [
    (1, 1, 1, 1, 64, 1, 0),          # single token
    (2, 77, 4, 2, 64, 5, 0),         # ragged T, small window, GQA 2
    (1, 130, 3, 1, 128, 33, 16),     # GQA 3, window not a multiple of anything
    (1, 200, 2, 2, 128, 64, 64),     # window = chunk
    (1, 150, 2, 1, 64, 1, 7),        # window 1 (softmax over the token itself), odd chunk
    (1, 96, 2, 2, 64, 96, 0),        # window = T: linear branch empty
    (1, 96, 2, 2, 64, 500, 0),       # window > T
    (2, 300, 4, 4, 128, 100, 100),   # long intra-chunk part (> 64 keys)
])
def test_fwd_f32_shapes(B, T, Hq, Hkv, D, W, chunk):
    run_fwd_case(B, T, Hq, Hkv, D, W, "f32", seed=100 + T, chunk=chunk, gains=True)


def test_fwd_f32_paper_formula_scale_one():
    run_fwd_case(1, 120, 2, 1, 64, 16, "f32", seed=5, scale=1.0, std=0.125)


@pytest.mark.parametrize("B,T,Hq,Hkv,D,W", [
    (1, 200, 4, 2, 128, 48),
    (2, 333, 2, 1, 64, 20),
    (1, 256, 2, 2, 128, 256),
])
def test_fwd_bf16_shapes(B, T, Hq, Hkv, D, W):
    run_fwd_case(B, T, Hq, Hkv, D, W, "bf16", seed=200 + T, gains=True)


def test_chunk_hint_does_not_change_result():
    x = synth.make_random_layer(1, 180, 2, 1, 64, "f32", 7)
    outs = [rb.rattn_fwd(dev(x["q"]), dev(x["k"]), dev(x["v"]), 20, chunk=c, softmax_scale=0.125) for c in (0, 16, 33, 128)]
    for o in outs[1:]:
        assert float((o - outs[0]).abs().max()) < 2e-5


def run_bwd_case(B, T, Hq, Hkv, D, W, dtype, seed, chunk=0, gains=True, kernel_path="auto"):
    x = synth.make_random_layer(B, T, Hq, Hkv, D, dtype, seed, with_dO=True, with_gains=gains)
    scale = 1.0 / math.sqrt(D)
    gs, gr = x.get("gamma_swa"), x.get("gamma_rla")
    print(f"bwd case B={B} T={T} Hq={Hq} Hkv={Hkv} D={D} W={W} {dtype} chunk={chunk} seed={seed}", flush=True)
    q, k, v, dO = dev(x["q"]), dev(x["k"]), dev(x["v"]), dev(x["dO"])
    o, saved = rb.rattn_fwd(q, k, v, W, dev(gs), dev(gr), chunk=chunk, softmax_scale=scale, save_for_bwd=True,
                            kernel_path=kernel_path)
    dq, dk, dv, dgs, dgr = rb.rattn_bwd(q, k, v, saved, dO, W, dev(gs), dev(gr), chunk=chunk, softmax_scale=scale,
                                        kernel_path=kernel_path)
    torch.cuda.synchronize()
    ref = orc.bwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), np64(x["dO"]), W, scale=scale,
                        gamma_swa=None if gs is None else np64(gs), gamma_rla=None if gr is None else np64(gr))
    tol = TOL[dtype]
    for name, got in (("dq", dq), ("dk", dk), ("dv", dv), ("dgamma_swa", dgs), ("dgamma_rla", dgr)):
        if np.all(ref[name] == 0):
            # an exactly-zero gradient (e.g. a one-key softmax) may come back as rounding noise
            assert float(got.abs().max()) <= tol * 1e-2, name
            continue
        e = rel_rms_err(got, ref[name], "f32" if name.startswith("dgamma") else dtype)
        assert e <= tol, f"{name}: rel err {e}"


@pytest.mark.parametrize("B,T,Hq,Hkv,D,W,chunk", [
    (1, 1, 1, 1, 64, 1, 0),
    (2, 77, 4, 2, 64, 5, 0),
    (1, 130, 3, 1, 128, 33, 16),
    (1, 150, 2, 1, 64, 1, 7),
    (1, 96, 2, 2, 64, 96, 0),
    (1, 260, 2, 2, 128, 70, 100),
])
def test_bwd_f32_shapes(B, T, Hq, Hkv, D, W, chunk):
    run_bwd_case(B, T, Hq, Hkv, D, W, "f32", seed=300 + T, chunk=chunk)


def test_bwd_config1_tiny_f32():
    cfg = synth.CONFIGS["tiny_f32"]
    q, k, v, dO = synth.make_layer_inputs(cfg, with_dO=True)
    o, saved = rb.rattn_fwd(q.cuda(), k.cuda(), v.cuda(), cfg.W, chunk=cfg.chunk, softmax_scale=cfg.scale, save_for_bwd=True)
    dq, dk, dv, _, _ = rb.rattn_bwd(q.cuda(), k.cuda(), v.cuda(), saved, dO.cuda(), cfg.W, chunk=cfg.chunk,
                                    softmax_scale=cfg.scale)
    ref = orc.bwd_dense(np64(q), np64(k), np64(v), np64(dO), cfg.W, scale=cfg.scale)
    for name, got in (("dq", dq), ("dk", dk), ("dv", dv)):
        assert rel_rms_err(got, ref[name]) <= 1e-4, name


@pytest.mark.parametrize("B,T,Hq,Hkv,D,W", [(1, 200, 4, 2, 128, 48), (2, 140, 2, 1, 64, 20),
                                              # windows of a few keys: near-one-hot softmax rows
                                              (2, 143, 3, 3, 128, 5), (2, 70, 6, 3, 128, 2), (1, 100, 2, 1, 64, 3)])
def test_bwd_bf16_shapes(B, T, Hq, Hkv, D, W):
    # the general kernels' bar (fp32 arithmetic): asked for explicitly where the shape would run on the matrix cores
    run_bwd_case(B, T, Hq, Hkv, D, W, "bf16", seed=400 + T, kernel_path="general")


# ------------------------------------------------------------------------------ decode
@pytest.mark.parametrize("dtype,D,Hq,Hkv,W,T", [("f32", 64, 4, 2, 8, 30), ("f32", 128, 3, 1, 5, 12),
                                                 ("bf16", 128, 8, 2, 16, 40), ("f32", 64, 6, 1, 50, 20)])
def test_decode_chain_reproduces_forward(dtype, D, Hq, Hkv, W, T):
    N = 3
    x = synth.make_random_layer(N, T, Hq, Hkv, D, dtype, 500 + T, with_gains=True)
    scale = 1.0 / math.sqrt(D)
    gs, gr = x["gamma_swa"], x["gamma_rla"]
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, scale=scale, gamma_swa=np64(gs), gamma_rla=np64(gr))["o"]
    dt = synth.torch_dtype(dtype)
    kr = torch.zeros(N, Hkv, W, D, dtype=dt, device="cuda"); vr = torch.zeros_like(kr)
    S = torch.zeros(N, Hkv, D, D, dtype=torch.float32, device="cuda")
    q, k, v = dev(x["q"]), dev(x["k"]), dev(x["v"])
    gmax = max(float(gs.abs().max()), float(gr.abs().max()), 1.0)
    for t in range(T):
        pos = torch.full((N,), t, dtype=torch.int32, device="cuda")
        o = rb.rattn_decode_step(q[:, t].contiguous(), k[:, t].contiguous(), v[:, t].contiguous(), pos, kr, vr, S,
                                 dev(gs), dev(gr), softmax_scale=scale)
        assert maxerr(o, ref[:, t]) <= TOL[dtype] * gmax, f"step {t}"
        assert torch.equal(kr[:, :, t % W], k[:, t])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_decode_step_random_positions(dtype):
    cfg = synth.DECODE_CONFIGS["decode_b128_w512"]
    cfg = synth.DecodeConfig("small", 6, 8, 2, 128, 64, dtype, 11, 0, 300, cfg.scale)
    pos = [0, 5, 63, 64, 65, 300]       # before the ring fills, at the edge, after
    x = synth.make_decode_inputs(cfg, pos=pos)
    o_ref, kr_ref, vr_ref, S_ref = orc.decode_step(np64(x["q"]), np64(x["k_new"]), np64(x["v_new"]), pos,
                                                   np64(x["k_ring"]), np64(x["v_ring"]), np64(x["state"]), cfg.W,
                                                   scale=cfg.scale)
    d = {k_: v_.cuda() for k_, v_ in x.items()}
    o = rb.rattn_decode_step(d["q"], d["k_new"], d["v_new"], d["pos"], d["k_ring"], d["v_ring"], d["state"],
                             softmax_scale=cfg.scale)
    assert maxerr(o, o_ref) <= TOL[dtype]
    assert np.array_equal(np64(d["k_ring"]), kr_ref) and np.array_equal(np64(d["v_ring"]), vr_ref)
    assert float(np.max(np.abs(np64(d["state"]) - S_ref))) <= 1e-5 * max(1.0, float(np.abs(S_ref).max()))


def _decode_vs_oracle(cfg, pos, tol):
    x = synth.make_decode_inputs(cfg, pos=pos)
    pos_l = [int(p) for p in x["pos"]]
    o_ref, kr_ref, vr_ref, S_ref = orc.decode_step(np64(x["q"]), np64(x["k_new"]), np64(x["v_new"]), pos_l,
                                                   np64(x["k_ring"]), np64(x["v_ring"]), np64(x["state"]), cfg.W,
                                                   scale=cfg.scale)
    d = {k_: v_.cuda() for k_, v_ in x.items()}
    o = rb.rattn_decode_step(d["q"], d["k_new"], d["v_new"], d["pos"], d["k_ring"], d["v_ring"], d["state"],
                             softmax_scale=cfg.scale)
    if cfg.dtype == "bf16":
        pm.assert_out_bf16(np64(o), o_ref, what=f"decode {cfg.name} o", tol=tol)
    else:
        assert float(np.abs(np64(o) - o_ref).max()) <= tol
    assert np.array_equal(np64(d["k_ring"]), kr_ref) and np.array_equal(np64(d["v_ring"]), vr_ref)
    assert float(np.max(np.abs(np64(d["state"]) - S_ref))) <= 1e-5 * max(1.0, float(np.abs(S_ref).max()))


@pytest.mark.parametrize("W", [200, 512, 1000])
def test_decode_bf16_long_rings(W):
    """Rings spanning several 128-key steps, a ragged last step, and every fill level of the ring."""
    cfg = synth.DecodeConfig("rings", 8, 8, 2, 128, W, "bf16", 13, 0, 4 * W, 1.0 / math.sqrt(128))
    pos = [0, 31, 127, 128, W - 1, W, W + 1, 3 * W + 77]
    _decode_vs_oracle(cfg, pos, TOL["bf16"])


def test_decode_full_config_all_sequences():
    """The decode workload the benchmark times (128 sequences, 32 query / 8 kv heads, W = 512), every output."""
    cfg = synth.DECODE_CONFIGS["decode_b128_w512"]
    _decode_vs_oracle(cfg, None, TOL["bf16"])


# ------------------------------------------------------------------------------ prefill -> decode hand-over
@pytest.mark.parametrize("dtype,B,T,Hkv,D,W", [("f32", 2, 5, 2, 64, 8), ("f32", 1, 8, 1, 64, 8), ("f32", 2, 77, 2, 128, 10),
                                                 ("bf16", 2, 384, 2, 128, 128), ("bf16", 1, 1000, 3, 64, 200),
                                                 ("bf16", 2, 2048, 2, 128, 512)])
def test_prefill_export_matches_oracle(dtype, B, T, Hkv, D, W):
    x = synth.make_random_layer(B, T, Hkv, Hkv, D, dtype, 800 + T)
    kr_ref, vr_ref, S_ref = orc.prefill_export(np64(x["k"]), np64(x["v"]), W)
    kr, vr, S = rb.rattn_prefill_export(dev(x["k"]), dev(x["v"]), W)
    assert np.array_equal(np64(kr), kr_ref) and np.array_equal(np64(vr), vr_ref)
    # fp32 sums of up to T-W exact products of a softmax row (fp32 exp) with a value
    assert float(np.max(np.abs(np64(S) - S_ref))) <= 2e-5 * max(1.0, float(np.abs(S_ref).max()))
    kr2, vr2, S2 = rb.rattn_prefill_export(dev(x["k"]), dev(x["v"]), W)
    assert torch.equal(S, S2)       # fixed summation order


@pytest.mark.parametrize("dtype,T,W", [("f32", 40, 16), ("bf16", 256, 64), ("bf16", 300, 512)])
def test_prefill_then_decode_reproduces_forward_row(dtype, T, W):
    """fwd over T+1 tokens, last row  ==  export(first T tokens) followed by one decode step at pos = T."""
    B, Hq, Hkv, D = 2, 4, 2, 128
    x = synth.make_random_layer(B, T + 1, Hq, Hkv, D, dtype, 850 + T, with_gains=True)
    scale = 1.0 / math.sqrt(D)
    gs, gr = x["gamma_swa"], x["gamma_rla"]
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, scale=scale, gamma_swa=np64(gs),
                        gamma_rla=np64(gr), rows=np.array([T]))["o"][:, T]
    q, k, v = dev(x["q"]), dev(x["k"]), dev(x["v"])
    kr, vr, S = rb.rattn_prefill_export(k[:, :T].contiguous(), v[:, :T].contiguous(), W)
    pos = torch.full((B,), T, dtype=torch.int32, device="cuda")
    o = rb.rattn_decode_step(q[:, T].contiguous(), k[:, T].contiguous(), v[:, T].contiguous(), pos, kr, vr, S,
                             dev(gs), dev(gr), softmax_scale=scale)
    gmax = max(float(gs.abs().max()), float(gr.abs().max()), 1.0)
    assert maxerr(o, ref) <= TOL[dtype] * gmax


@pytest.mark.parametrize("dtype,D,Hq,Hkv,W,chunks", [
    ("f32", 64, 4, 2, 8, [5, 3, 9, 1, 12]),          # history shorter than, equal to and longer than the window
    ("f32", 128, 2, 1, 16, [16, 16, 7]),
    ("f32", 64, 2, 2, 4, [1, 1, 1, 1, 1, 1, 3]),     # single-token chunks = decode steps
    ("bf16", 128, 4, 2, 128, [128, 256, 128]),       # ring + chunk a multiple of 128: matrix-core kernels
    ("bf16", 128, 2, 2, 256, [128, 384, 256, 128]),  # history shorter than the window in whole tiles, then longer
    ("bf16", 128, 2, 1, 192, [192, 192, 256]),       # window no multiple of 128: gather + fix-up route
    ("bf16", 128, 2, 1, 513, [640, 255, 383]),       # the same with a window that is no tile multiple
    ("bf16", 64, 3, 1, 50, [70, 130]),
    ("bf16", 128, 2, 1, 100, [1100, 500]),           # ring + chunk >= 1024, not a multiple of 128: padded copies
])
def test_chunked_prefill_reproduces_forward(dtype, D, Hq, Hkv, W, chunks):
    """A prompt fed in chunks through rattn_prefill_chunk gives the rows of the forward over the whole prompt
    (oracle, fp64), and leaves the rings and the state the oracle's export gives for the whole prompt."""
    B, T = 2, sum(chunks)
    x = synth.make_random_layer(B, T, Hq, Hkv, D, dtype, 4100 + T + W, with_gains=True)
    scale = 1.0 / math.sqrt(D)
    gs, gr = x["gamma_swa"], x["gamma_rla"]
    ref = orc.fwd_dense(np64(x["q"]), np64(x["k"]), np64(x["v"]), W, scale=scale, gamma_swa=np64(gs),
                        gamma_rla=np64(gr))["o"]
    kr_ref, vr_ref, S_ref = orc.prefill_export(np64(x["k"]), np64(x["v"]), W)
    q, k, v = dev(x["q"]), dev(x["k"]), dev(x["v"])
    kr = torch.zeros(B, Hkv, W, D, dtype=q.dtype, device="cuda")
    vr = torch.zeros_like(kr)
    S = torch.full((B, Hkv, D, D), float("nan"), dtype=torch.float32, device="cuda")  # not read before pos0 > W
    gmax = max(float(gs.abs().max()), float(gr.abs().max()), 1.0)
    pos0 = 0
    for n in chunks:
        print(f"chunked prefill {dtype} D={D} W={W}: tokens {pos0}..{pos0 + n - 1}", flush=True)
        sl = slice(pos0, pos0 + n)
        o = rb.rattn_prefill_chunk(q[:, sl].contiguous(), k[:, sl].contiguous(), v[:, sl].contiguous(), W, pos0, kr, vr,
                                   S, dev(gs), dev(gr), softmax_scale=scale)
        torch.cuda.synchronize()
        r = ref[:, sl]
        if dtype == "bf16":
            pm.assert_out_bf16(np64(o), r, gmax, what=f"chunk at {pos0}")
        else:
            assert float(np.abs(np64(o) - r).max()) <= TOL[dtype] * gmax, pos0
        pos0 += n
    assert np.array_equal(np64(kr), kr_ref) and np.array_equal(np64(vr), vr_ref)
    assert float(np.max(np.abs(np64(S) - S_ref))) <= 2e-5 * max(1.0, float(np.abs(S_ref).max()))


def test_chunked_prefill_uses_matrix_core_kernels():
    B, Hq, Hkv, D, W = 1, 2, 1, 128, 128
    x = synth.make_random_layer(B, 384, Hq, Hkv, D, "bf16", 4200)
    q, k, v = dev(x["q"]), dev(x["k"]), dev(x["v"])
    kr, vr, S = rb.rattn_prefill_export(k[:, :256].contiguous(), v[:, :256].contiguous(), W)
    rb.rattn_profile_enable(True)
    rb.rattn_prefill_chunk(q[:, 256:].contiguous(), k[:, 256:].contiguous(), v[:, 256:].contiguous(), W, 256, kr, vr, S,
                           softmax_scale=0.09)
    torch.cuda.synchronize()
    names = [n for n, _ in rb.rattn_profile_records()]
    rb.rattn_profile_enable(False)
    # whole tiles of ring and chunk, window a multiple of 128: the forward runs on the chunk's query tiles only and
    # takes the carried state as the start of its state scan; nothing is fixed up or copied afterwards
    assert "fwd_fused_kernel" in names and "gen_fwd_kernel" not in names
    assert "chunk_fixup_kernel" not in names and "chunk_copy_out_kernel" not in names
    # a window that is no multiple of 128 leaves a first tile without a chunk state: gather + fix-up route
    x = synth.make_random_layer(B, 704, Hq, Hkv, D, "bf16", 4201)      # ring 192 + chunk 320 = 512 rows
    q, k, v = dev(x["q"]), dev(x["k"]), dev(x["v"])
    kr, vr, S = rb.rattn_prefill_export(k[:, :384].contiguous(), v[:, :384].contiguous(), 192)
    rb.rattn_profile_enable(True)
    rb.rattn_prefill_chunk(q[:, 384:].contiguous(), k[:, 384:].contiguous(), v[:, 384:].contiguous(), 192, 384, kr, vr, S,
                           softmax_scale=0.09)
    torch.cuda.synchronize()
    names = [n for n, _ in rb.rattn_profile_records()]
    rb.rattn_profile_enable(False)
    assert "fwd_fused_kernel" in names and "chunk_fixup_kernel" in names
