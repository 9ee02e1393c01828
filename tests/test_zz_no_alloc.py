"""The allocation-free forward entry point (rattn_fwd_static: scratch inside the library's device image) against
rattn_fwd with a caller-provided workspace, through the C ABI: two calls in a row, the second on a smaller input
(it reuses the front of the buffer the first call left dirty), then a ragged length that runs through padded
copies in the scratch, and the size limit."""
import ctypes
import math
import pytest
import torch

from paper_2506_15545_amd import binding as rb
from paper_2506_15545_amd import synth


def _params(B, T, Hq, Hkv, D, W):
    return rb.RattnParams(B, T, Hq, Hkv, D, W, 0, rb.RATTN_BF16, 1.0 / math.sqrt(D), 1e-6, 0, 0, 0, 0)


def test_static_entry_rejects_shapes_beyond_its_buffer():
    # host-side check only: nothing is launched and no device is touched before the size test
    p = _params(4, 8192, 24, 8, 128, 512)
    fwd_b, _, _ = rb.rattn_workspace_bytes(p)
    assert fwd_b > rb.STATIC_SCRATCH_BYTES
    st = rb.lib().rattn_fwd_static(ctypes.byref(p), *([None] * 8))
    assert st == -3 and b"built-in buffer" in rb.lib().rattn_last_error()
    p.T = 0
    assert rb.lib().rattn_fwd_static(ctypes.byref(p), *([None] * 8)) == -1


@pytest.mark.gpu
def test_static_entry_matches_workspace_entry_on_two_calls_in_a_row():
    torch.cuda.set_device(0)
    cases = [
        (2, 2048, 8, 2, 128, 256, 31),    # matrix-core path, 14 chunk states per KV head
        (1, 640, 4, 2, 128, 192, 32),     # smaller: reuses the front of the dirty buffer; states at the 64 alignment
        (1, 1100, 2, 1, 128, 300, 33),    # ragged length: the tail buffers of q, k, v, o live in the scratch too
        (1, 100, 4, 2, 64, 32, 34),       # general kernels (less than one tile): fp32 chunk states in the scratch
    ]
    for (B, T, Hq, Hkv, D, W, seed) in cases:
        print(f"static entry case B={B} T={T} Hq={Hq} Hkv={Hkv} D={D} W={W}", flush=True)
        x = synth.make_random_layer(B, T, Hq, Hkv, D, "bf16", seed, with_gains=True)
        q, k, v = x["q"].cuda(), x["k"].cuda(), x["v"].cuda()
        gs, gr = x["gamma_swa"].cuda(), x["gamma_rla"].cuda()
        scale = 1.0 / math.sqrt(D)
        p = rb.make_params(q, k, W, 0, scale, 1e-6, True)
        fwd_b, _, saved_b = rb.rattn_workspace_bytes(p)
        assert fwd_b <= rb.STATIC_SCRATCH_BYTES
        o_ref, saved_ref = rb.rattn_fwd(q, k, v, W, gs, gr, softmax_scale=scale, save_for_bwd=True)
        o = torch.full_like(q, float("nan"))
        saved = torch.zeros(saved_b, dtype=torch.uint8, device="cuda")
        before = torch.cuda.memory_allocated()
        rb.rattn_fwd_static(q, k, v, W, o, gs, gr, softmax_scale=scale, saved=saved)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        # same kernels on the same inputs: the bits agree (stronger than the parity tolerance)
        assert torch.equal(o, o_ref)
        n = B * T * Hq * D * (2 if T >= 128 else 4)
        if T % 128 == 0 or T < 128:  # pre-norm output of the softmax branch (ragged lengths: laid out for the padded T)
            assert torch.equal(saved[:n], saved_ref[:n])
        # and without saving
        o2 = torch.full_like(q, float("nan"))
        rb.rattn_fwd_static(q, k, v, W, o2, gs, gr, softmax_scale=scale)
        torch.cuda.synchronize()
        assert torch.equal(o2, o_ref)
