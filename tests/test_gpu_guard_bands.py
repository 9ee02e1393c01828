"""Out-of-bounds writes: every buffer the library writes (outputs, `saved`, workspace, gradients, rings, state) is
carved out of a larger allocation with 4 KiB of a known byte pattern in front of and behind it; after the call the
pattern must be intact.  Shapes: a 3B-layer-shaped case, a ragged length (tail buffers in the workspace), windows that
are no tile multiples (the extra key tile of the linear branch), the general kernels, chunked prefill on both routes,
prefill export and decode.  Nothing here provokes a fault: all sizes are the ones the library itself reports."""
import ctypes
import math

import pytest
import torch

from paper_2506_15545_amd import binding as rb
from paper_2506_15545_amd import synth

pytestmark = pytest.mark.gpu

GUARD = 4096
PATTERN = 0xA5


class Guarded:
    """`nbytes` of device memory (256-byte aligned) with GUARD bytes of PATTERN on both sides."""

    def __init__(self, nbytes, name):
        self.name = name
        self.n = int(nbytes)
        pad = (-self.n) % 256
        self.full = torch.full((GUARD + self.n + pad + GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        self.bytes = self.full[GUARD:GUARD + self.n]
        self.tail0 = GUARD + self.n

    def view(self, dtype, shape):
        return self.bytes.view(dtype).view(shape)

    def check(self):
        front = self.full[:GUARD]
        back = self.full[self.tail0:]
        assert bool((front == PATTERN).all()), f"{self.name}: bytes in front of the buffer were overwritten"
        assert bool((back == PATTERN).all()), f"{self.name}: bytes behind the buffer were overwritten"


def guarded_like(t, name):
    g = Guarded(t.numel() * t.element_size(), name)
    return g, g.view(t.dtype, t.shape)


LAYER_CASES = [
    # B, T, Hq, Hkv, D, W, dtype, path
    (1, 1024, 6, 2, 128, 512, "bf16", "auto"),     # the benchmark layer's head ratio and window
    (2, 1100, 2, 1, 128, 300, "bf16", "auto"),     # ragged: the last partial tile of q, k, v, o, dO, dq, dk, dv goes through the workspace
    (1, 640, 4, 2, 128, 513, "bf16", "auto"),      # window = 512 earlier tokens + the current one
    (1, 384, 3, 1, 128, 100, "bf16", "auto"),      # gap > 0, states at the 64 alignment
    (2, 300, 2, 1, 128, 77, "bf16", "auto"),       # short ragged length, gap > 0: tail buffers
    (1, 256, 2, 1, 128, 250, "bf16", "auto"),      # window rounds up to T
    (1, 384, 2, 2, 128, 1000, "bf16", "auto"),     # causal: no linear branch, no states
    (2, 100, 4, 2, 64, 32, "bf16", "auto"),        # general kernels (less than one tile)
    (2, 200, 4, 2, 64, 32, "bf16", "auto"),        # head size 64, ragged and short: widened copies
    (1, 256, 4, 2, 64, 100, "bf16", "auto"),       # head size 64 on the matrix-core kernels: widened copies, gains too
    (1, 1030, 2, 1, 64, 200, "bf16", "auto"),      # head size 64 and a ragged length together
    (1, 300, 2, 1, 128, 77, "f32", "auto"),        # general kernels, fp32
    (1, 512, 4, 2, 128, 128, "bf16", "general"),   # general kernels forced on a matrix-core shape
]


@pytest.mark.parametrize("B,T,Hq,Hkv,D,W,dtype,path", LAYER_CASES)
def test_layer_calls_stay_inside_their_buffers(B, T, Hq, Hkv, D, W, dtype, path):
    print(f"guard bands: B={B} T={T} Hq={Hq} Hkv={Hkv} D={D} W={W} {dtype} {path}", flush=True)
    x = synth.make_random_layer(B, T, Hq, Hkv, D, dtype, 4000 + T + W, with_dO=True, with_gains=True)
    q, k, v, dO = (x[n].cuda() for n in ("q", "k", "v", "dO"))
    gs, gr = x["gamma_swa"].cuda(), x["gamma_rla"].cuda()
    scale = 1.0 / math.sqrt(D)
    p = rb.make_params(q, k, W, 0, scale, 1e-6, True, "softmax", path)
    fwd_b, bwd_b, saved_b = rb.rattn_workspace_bytes(p)
    ws_f, ws_b, sv = Guarded(max(fwd_b, 16), "forward workspace"), Guarded(max(bwd_b, 16), "backward workspace"), \
        Guarded(saved_b, "saved")
    go, o = guarded_like(q, "o")
    gdq, dq = guarded_like(q, "dq")
    gdk, dk = guarded_like(k, "dk")
    gdv, dv = guarded_like(v, "dv")
    rb.rattn_fwd(q, k, v, W, gs, gr, softmax_scale=scale, save_for_bwd=True, out=o, saved=sv.bytes, workspace=ws_f.bytes,
                 kernel_path=path)
    _, _, _, dgs, dgr = rb.rattn_bwd(q, k, v, sv.bytes, dO, W, gs, gr, softmax_scale=scale, workspace=ws_b.bytes,
                                     out=(dq, dk, dv), kernel_path=path)
    torch.cuda.synchronize()
    for g in (ws_f, ws_b, sv, go, gdq, gdk, gdv):
        g.check()
    assert torch.isfinite(o.float()).all() and torch.isfinite(dq.float()).all()
    # forward without saving: `saved` may be NULL and must not be touched
    go2, o2 = guarded_like(q, "o (no save)")
    rb.rattn_fwd(q, k, v, W, gs, gr, softmax_scale=scale, out=o2, workspace=ws_f.bytes, kernel_path=path)
    torch.cuda.synchronize()
    go2.check(); ws_f.check()
    assert torch.equal(o, o2)


@pytest.mark.parametrize("D,Hq,Hkv,W,chunks", [
    (128, 4, 2, 128, [256, 128, 128]),     # direct route on the matrix-core kernels, carried state
    (128, 2, 1, 100, [200, 56, 300]),      # gather route, windows and histories that are no tile multiples
    (64, 2, 2, 16, [40, 3, 21]),           # general kernels
])
def test_chunked_prefill_export_and_decode_stay_inside_their_buffers(D, Hq, Hkv, W, chunks):
    B, T = 2, sum(chunks)
    print(f"guard bands, chunked prefill: D={D} Hq={Hq} Hkv={Hkv} W={W} chunks={chunks}", flush=True)
    x = synth.make_random_layer(B, T, Hq, Hkv, D, "bf16", 4100 + W)
    q, k, v = x["q"].cuda(), x["k"].cuda(), x["v"].cuda()
    scale = 1.0 / math.sqrt(D)
    gkr, kr = guarded_like(torch.empty(B, Hkv, W, D, dtype=torch.bfloat16), "k_ring")
    gvr, vr = guarded_like(torch.empty(B, Hkv, W, D, dtype=torch.bfloat16), "v_ring")
    gst, S = guarded_like(torch.empty(B, Hkv, D, D, dtype=torch.float32), "state")
    kr.zero_(); vr.zero_(); S.zero_()
    pos0 = 0
    for n in chunks:
        sl = slice(pos0, pos0 + n)
        qc, kc, vc = q[:, sl].contiguous(), k[:, sl].contiguous(), v[:, sl].contiguous()
        p = rb.make_params(qc, kc, W, 0, scale, 1e-6, False)
        nb = ctypes.c_size_t()
        assert rb.lib().rattn_prefill_chunk_workspace_bytes(ctypes.byref(p), pos0, ctypes.byref(nb)) == 0
        ws = Guarded(max(nb.value, 16), f"chunk workspace at {pos0}")
        go, o = guarded_like(qc, f"chunk o at {pos0}")
        rb.rattn_prefill_chunk(qc, kc, vc, W, pos0, kr, vr, S, softmax_scale=scale, workspace=ws.bytes, out=o)
        torch.cuda.synchronize()
        for g in (ws, go, gkr, gvr, gst):
            g.check()
        pos0 += n
    # prefill export over the whole prompt into fresh guarded rings / state
    gkr2, kr2 = guarded_like(kr, "exported k_ring")
    gvr2, vr2 = guarded_like(vr, "exported v_ring")
    gst2, S2 = guarded_like(S, "exported state")
    kr2.zero_(); vr2.zero_()
    rb.rattn_prefill_export(k, v, W, kr2, vr2, S2)
    torch.cuda.synchronize()
    for g in (gkr2, gvr2, gst2):
        g.check()
    assert torch.equal(kr, kr2) and torch.equal(vr, vr2)
    # one decode step on top
    g_ = torch.Generator().manual_seed(5)
    qn = torch.randn(B, Hq, D, generator=g_).to(torch.bfloat16).cuda()
    kn = torch.randn(B, Hkv, D, generator=g_).to(torch.bfloat16).cuda()
    vn = torch.randn(B, Hkv, D, generator=g_).to(torch.bfloat16).cuda()
    pos = torch.full((B,), T, dtype=torch.int32, device="cuda")
    god, od = guarded_like(qn, "decode o")
    rb.rattn_decode_step(qn, kn, vn, pos, kr2, vr2, S2, softmax_scale=scale, out=od)
    torch.cuda.synchronize()
    for g in (god, gkr2, gvr2, gst2):
        g.check()


def test_decode_config_shape_stays_inside_its_buffers():
    cfg = synth.DecodeConfig("guard", 16, 32, 8, 128, 512, "bf16", 21, 0, 4096, 1.0 / math.sqrt(128))
    d = synth.make_decode_inputs(cfg)
    gk, kr = guarded_like(d["k_ring"], "k_ring")
    gv, vr = guarded_like(d["v_ring"], "v_ring")
    gs_, S = guarded_like(d["state"], "state")
    kr.copy_(d["k_ring"]); vr.copy_(d["v_ring"]); S.copy_(d["state"])
    go, o = guarded_like(d["q"], "o")
    rb.rattn_decode_step(d["q"].cuda(), d["k_new"].cuda(), d["v_new"].cuda(), d["pos"].cuda(), kr, vr, S,
                         softmax_scale=cfg.scale, out=o)
    torch.cuda.synchronize()
    for g in (gk, gv, gs_, go):
        g.check()
