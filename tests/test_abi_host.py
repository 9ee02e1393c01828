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
             rms_eps=1e-6, save_for_bwd=0, feature_map=0, kernel_path=0, state_policy=0)
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
    (dict(feature_map=3), -2), (dict(feature_map=-1), -2), (dict(kernel_path=2), -2), (dict(state_policy=3), -2), (dict(state_policy=-1), -2),
    (dict(B=60000, T=10000), -2),      # more rows than 32-bit row indexing covers
    (dict(B=70000), -2), (dict(Hq=70000, Hkv=70000), -2),   # grid dimensions
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
    dp.D = 64
    dp.N = 70000
    assert L.rattn_decode_step(ctypes.byref(dp), *([None] * 11)) == -2 and b"N must be" in L.rattn_last_error()
    dp.N = 4
    dp.feature_map = 5
    assert L.rattn_decode_step(ctypes.byref(dp), *([None] * 11)) == -2 and b"feature_map" in L.rattn_last_error()


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


def test_inference_closed_forms_match_the_oracle_and_the_text():
    """rattn_cache_bytes / rattn_step_time_model (host arithmetic) against the oracle's closed forms, and against
    what the text says: ~56 % cache saving for the 12B stack at 4K context when the local window shrinks from 4K
    to 1K (Sec. 1), and a step-time gain that grows with the batch towards roughly 60 % and depends on the cache
    ratio alone, not on the model size, once the cache dominates (Sec. 4.4: window 512 against sliding-window 4K, H100 figures, bf16)."""
    import random
    from oracle import rattn_oracle as orc
    # cache of a local-global stack without state = the oracle's token count times the bytes of a token
    big = rb.rattn_cache_bytes(40, 4, 4096, 4096, False, 8, 128, 2)
    small = rb.rattn_cache_bytes(40, 4, 4096, 1024, False, 8, 128, 2)
    assert abs((1.0 - small / big) - orc.kv_cache_saving(40, 4, 4096, 4096, 1024)) < 1e-12
    assert abs((1.0 - small / big) - 0.5625) < 1e-12
    assert big == 40 * 4096 * 2 * 8 * 128 * 2
    # the fp32 D x D state of a local layer = twice the bf16 window-equivalent of the text's footnote (64 tokens)
    with_state = rb.rattn_cache_bytes(40, 4, 4096, 1024, True, 8, 128, 2)
    per_state = (with_state - small) / (30 * 8)
    assert per_state == 2 * orc.state_equivalent_window(128, 128) * 2 * 128 * 2
    # a context shorter than the window caps the local layers; no global layers when global_every = 0
    assert rb.rattn_cache_bytes(8, 0, 100, 512, False, 2, 64, 4) == 8 * 100 * 2 * 2 * 64 * 4
    rng = random.Random(5)
    for _ in range(50):
        a = [rng.uniform(0, 1e3), rng.uniform(0, 1e9), rng.uniform(0, 1e11), rng.uniform(0, 1e11), rng.uniform(1e9, 1e13),
             rng.uniform(1e12, 1e16)]
        assert abs(rb.rattn_step_time_model(*a) - orc.decode_step_time(*a)) <= 1e-12 * orc.decode_step_time(*a)
    # Sec. 4.4 case study: H100 (3.35 TB/s, 989 TFLOP/s dense bf16), 3:1 local:global stacks
    bw, fl = 3.35e12, 989e12
    models = {"3B": (56, 4, 3e9), "12B": (40, 8, 12e9)}

    def gain(name, batch, ctx):
        layers, hkv, pc = models[name]
        swa = rb.rattn_cache_bytes(layers, 4, ctx, 4096, False, hkv, 128, 2)
        ratt = rb.rattn_cache_bytes(layers, 4, ctx, 512, True, hkv, 128, 2)
        t0 = rb.rattn_step_time_model(batch, swa, pc, 2 * pc, bw, fl)
        t1 = rb.rattn_step_time_model(batch, ratt, pc, 2 * pc, bw, fl)
        return 1.0 - t1 / t0

    for name in models:
        g = [gain(name, b, 4096) for b in (1, 8, 64, 512, 4096)]
        assert all(x <= y for x, y in zip(g, g[1:])) and g[0] < 0.1 < g[2]   # grows with the batch, then saturates
        assert 0.55 < g[-1] < 0.66                                           # "up to approximately 60 %"
    # where the cache is all that matters (no parameter terms) the gain is the cache ratio alone, whatever the model
    lim = {}
    for name, (layers, hkv, pc) in models.items():
        swa = rb.rattn_cache_bytes(layers, 4, 4096, 4096, False, hkv, 128, 2)
        ratt = rb.rattn_cache_bytes(layers, 4, 4096, 512, True, hkv, 128, 2)
        lim[name] = 1.0 - rb.rattn_step_time_model(1e6, ratt, 0.0, 0.0, bw, fl) / rb.rattn_step_time_model(1e6, swa, 0.0, 0.0, bw, fl)
        assert gain(name, 4096, 4096) < lim[name]
    assert abs(lim["3B"] - lim["12B"]) < 1e-12 and abs(lim["3B"] - (1.0 - (3 * 640 + 4096) / (4 * 4096))) < 1e-12
    assert gain("12B", 4096, 131072) < gain("12B", 4096, 4096)                  # global layers dominate long contexts
    out = ctypes.c_double()
    assert rb.lib().rattn_step_time_model(1.0, 1.0, 1.0, 1.0, 0.0, 1.0, ctypes.byref(out)) == -1
    assert rb.lib().rattn_cache_bytes(4, 4, -1, 8, 0, 1, 64, 2, ctypes.byref(out)) == -1
    assert rb.lib().rattn_cache_bytes(4, 4, 1, 8, 0, 1, 64, 2, None) == -1


def test_matrix_core_chunk_size_defaults_to_128_keys():
    """On the matrix-core path the chunk products cover 128 keys unless the caller asks for 64 (then there are twice
    as many, and the forward scratch that holds them doubles); other values mean 128."""
    base = dict(B=2, T=2048, Hq=4, Hkv=2, D=128, window=256, dtype=rb.RATTN_BF16)
    f0, _, _ = rb.rattn_workspace_bytes(params(**base))
    f64, _, _ = rb.rattn_workspace_bytes(params(chunk=64, **base))
    f128, _, _ = rb.rattn_workspace_bytes(params(chunk=128, **base))
    f32, _, _ = rb.rattn_workspace_bytes(params(chunk=32, **base))
    nst = 2048 // 128 - 2
    state_bytes = 2 * 2 * nst * 128 * 128 * 2
    assert f0 == f128 == f32 == 2 * 2 * (nst - 1) * 128 * 128 * 4 + state_bytes
    assert f64 == 2 * 2 * 2 * (nst - 1) * 128 * 128 * 4 + state_bytes
    # keeping no states for backward shrinks `saved` by exactly the states
    _, _, s_keep = rb.rattn_workspace_bytes(params(**base))
    _, _, s_rebuild = rb.rattn_workspace_bytes(params(state_policy=1, **base))
    assert s_keep - s_rebuild == state_bytes
    # every 2nd / 4th state kept (states 0, m, 2m, ...)
    _, _, s2 = rb.rattn_workspace_bytes(params(state_policy=2, **base))
    _, _, s4 = rb.rattn_workspace_bytes(params(state_policy=4, **base))
    assert s2 - s_rebuild == state_bytes // nst * ((nst + 1) // 2)
    assert s4 - s_rebuild == state_bytes // nst * ((nst + 3) // 4)


def test_ragged_lengths_cost_tail_buffers_not_copies():
    """A bf16, D = 128 length that is no multiple of 128 runs in place on the matrix-core kernels: on top of the
    scratch of the length rounded up, the workspace holds one 128-row buffer per tensor that passes through the
    kernels (forward q, k, v, o; backward q, k, v, dO, dq, dk, dv) and `saved` is that of the rounded-up length.
    A head size of 64 pays whole widened copies instead; lengths below one tile stay on the general kernels."""
    B, Hq, Hkv = 2, 6, 2
    base = dict(B=B, Hq=Hq, Hkv=Hkv, D=128, window=256, dtype=rb.RATTN_BF16)
    f_al, b_al, s_al = rb.rattn_workspace_bytes(params(T=2048, **base))
    f_rg, b_rg, s_rg = rb.rattn_workspace_bytes(params(T=2000, **base))
    tail_q, tail_kv = B * 128 * Hq * 128 * 2, B * 128 * Hkv * 128 * 2
    gains = 2 * Hq * 128 * 4                        # two widened gain rows per head (used at D = 64 only)
    assert s_rg == s_al
    assert f_rg == f_al + 2 * tail_q + 2 * tail_kv + gains
    assert b_rg == b_al + 3 * tail_q + 4 * tail_kv + 2 * gains
    # D = 64: whole tensors, widened to 128 features, forward and backward
    f64, b64, _ = rb.rattn_workspace_bytes(params(T=2048, **dict(base, D=64)))
    full_q, full_kv = B * 2048 * Hq * 128 * 2, B * 2048 * Hkv * 128 * 2
    assert f64 == f_al + 2 * full_q + 2 * full_kv + gains
    assert b64 == b_al + 3 * full_q + 4 * full_kv + 2 * gains
    # less than one tile: general kernels (fp32 branch outputs in `saved`)
    _, _, s_small = rb.rattn_workspace_bytes(params(T=100, **base))
    assert s_small >= 2 * B * 100 * Hq * 128 * 4
