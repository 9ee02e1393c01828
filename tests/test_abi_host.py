"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, reports workspace sizes and rejects bad arguments before launching."""
import ctypes
import os
import re
import pytest

from paper_2506_15545_amd import binding as rb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rattn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = rb.lib()
    names = declared_symbols()
    assert set(names) == set(rb.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert L.rattn_version().decode()
    assert L.rattn_status_string(0) == b"ok"


def params(**kw):
    d = dict(B=2, T=300, Hq=4, Hkv=2, D=64, window=32, chunk=0, dtype=rb.RATTN_F32, softmax_scale=1.0,
             rms_eps=1e-6, save_for_bwd=0)
    d.update(kw)
    return rb.RattnParams(**d)


def test_workspace_sizes_scale_with_shape():
    f1, b1, s1 = rb.rattn_workspace_bytes(params())
    f2, b2, s2 = rb.rattn_workspace_bytes(params(B=4))
    assert f1 > 0 and b1 > f1 and s1 > 0
    assert f2 >= 2 * f1 - 1024 and s2 >= 2 * s1 - 4096
    # saved holds two [B,T,Hq,D] tensors in the I/O dtype plus three fp32 row statistics
    assert s1 >= 2 * 2 * 300 * 4 * 64 * 4 + 3 * 2 * 4 * 300 * 4
    # window covering the sequence: no linear-branch states are needed
    f3, _, _ = rb.rattn_workspace_bytes(params(window=300))
    assert f3 == 0


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), -1), (dict(T=0), -1), (dict(Hq=3, Hkv=2), -1), (dict(window=0), -1), (dict(chunk=-1), -1),
    (dict(rms_eps=0.0), -1), (dict(softmax_scale=0.0), -1), (dict(D=96), -2), (dict(dtype=7), -2),
])
def test_bad_params_rejected(kw, code):
    with pytest.raises(rb.RattnError) as e:
        rb.rattn_workspace_bytes(params(**kw))
    assert e.value.status == code
    assert e.value.detail


def test_null_pointers_rejected_before_any_launch():
    L = rb.lib()
    p = params()
    st = L.rattn_fwd(ctypes.byref(p), None, None, None, None, None, None, None, None, 0, None)
    assert st == -1 and b"non-NULL" in L.rattn_last_error()
    st = L.rattn_bwd(ctypes.byref(p), *([None] * 13), 0, None)
    assert st == -1
    dp = rb.RattnDecodeParams(4, 4, 2, 64, 16, rb.RATTN_BF16, 1.0, 1e-6)
    st = L.rattn_decode_step(ctypes.byref(dp), *([None] * 11))
    assert st == -1
    dp.D = 80
    assert L.rattn_decode_step(ctypes.byref(dp), *([None] * 11)) == -2


def test_small_workspace_rejected():
    L = rb.lib()
    p = params()
    fake = ctypes.c_void_p(4096)  # never dereferenced: the size check fails first
    st = L.rattn_fwd(ctypes.byref(p), fake, fake, fake, None, None, fake, None, fake, 16, None)
    assert st == -3 and b"workspace" in L.rattn_last_error()
    st = L.rattn_fwd(ctypes.byref(p), ctypes.c_void_p(4097), fake, fake, None, None, fake, None, fake, 1 << 40, None)
    assert st == -1 and b"aligned" in L.rattn_last_error()


def test_prefill_export_host_checks():
    L = rb.lib()
    p = params()
    n = ctypes.c_size_t()
    assert L.rattn_prefill_export_workspace_bytes(ctypes.byref(p), ctypes.byref(n)) == 0
    # one fp32 D x D partial state per (batch row, kv head, key segment)
    assert n.value > 0 and n.value % (p.B * p.Hkv * p.D * p.D * 4) == 0
    fake = ctypes.c_void_p(4096)  # never dereferenced: the checks below fail first
    assert L.rattn_prefill_export(ctypes.byref(p), None, None, None, None, None, None, 0, None) == -1
    st = L.rattn_prefill_export(ctypes.byref(p), fake, fake, fake, fake, fake, fake, 16, None)
    assert st == -3 and b"workspace" in L.rattn_last_error()
    st = L.rattn_prefill_export(ctypes.byref(p), ctypes.c_void_p(4100), fake, fake, fake, fake, fake, 1 << 40, None)
    assert st == -1 and b"aligned" in L.rattn_last_error()
    # a prompt shorter than the window has no state to build: no scratch needed
    q = params(window=1000)
    assert L.rattn_prefill_export_workspace_bytes(ctypes.byref(q), ctypes.byref(n)) == 0 and n.value == 0


def test_prefill_chunk_host_checks():
    L = rb.lib()
    p = params()
    n0, n1 = ctypes.c_size_t(), ctypes.c_size_t()
    assert L.rattn_prefill_chunk_workspace_bytes(ctypes.byref(p), 0, ctypes.byref(n0)) == 0
    assert L.rattn_prefill_chunk_workspace_bytes(ctypes.byref(p), 10 * p.window, ctypes.byref(n1)) == 0
    # with a history the forward also runs over the ring rows: more scratch, and no more than for a full ring
    assert n1.value > n0.value > 0
    n2 = ctypes.c_size_t()
    assert L.rattn_prefill_chunk_workspace_bytes(ctypes.byref(p), p.window, ctypes.byref(n2)) == 0 and n2.value == n1.value
    assert L.rattn_prefill_chunk_workspace_bytes(ctypes.byref(p), -1, ctypes.byref(n0)) == -1
    fake = ctypes.c_void_p(4096)  # never dereferenced: the checks below fail first
    args = [fake] * 3 + [None, None] + [fake] * 4
    assert L.rattn_prefill_chunk(ctypes.byref(p), 0, *([None] * 9), None, 0, None) == -1
    st = L.rattn_prefill_chunk(ctypes.byref(p), 0, *args, fake, 16, None)
    assert st == -3 and b"workspace" in L.rattn_last_error()
    bad = [ctypes.c_void_p(4100)] + args[1:]
    st = L.rattn_prefill_chunk(ctypes.byref(p), 0, *bad, fake, 1 << 40, None)
    assert st == -1 and b"aligned" in L.rattn_last_error()
