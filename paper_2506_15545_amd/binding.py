"""ctypes binding of librattn.so: same entry-point names as include/rattn.h.

Only argument marshalling happens here (shape checks, buffer allocation through torch,
raw device pointers, the current HIP stream).  Every arithmetic step of the layer runs in
the library's kernels; there is no fallback: a missing library raises.
"""
import ctypes
import os
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librattn.so")

RATTN_F32, RATTN_BF16 = 0, 1
# rattn_feature_map: the layer's softmax map (Sec. 3.1) and the ablation's two alternatives (Sec. 4.5)
FEATURE_MAPS = {"softmax": 0, "relu": 1, "identity": 2}
# rattn_kernel_path: "auto" lets the library choose, "general" forces the general kernels (tests)
KERNEL_PATHS = {"auto": 0, "general": 1}
# rattn_state_policy: keep the chunk states in `saved` for backward (all, every 2nd, every 4th), or rebuild them
# there (Sec. 3.2 trade-off)
STATE_POLICIES = {"keep": 0, "rebuild": 1, "every2": 2, "every4": 4}
_DTYPES = {torch.float32: RATTN_F32, torch.bfloat16: RATTN_BF16}

EXPORTS = ["rattn_workspace_bytes", "rattn_fwd", "rattn_fwd_static", "rattn_bwd", "rattn_decode_step",
           "rattn_prefill_export_workspace_bytes", "rattn_prefill_export",
           "rattn_prefill_chunk_workspace_bytes", "rattn_prefill_chunk", "rattn_probe_mfma",
           "rattn_cache_bytes", "rattn_step_time_model",
           "rattn_status_string", "rattn_last_error", "rattn_version",
           "rattn_profile_enable", "rattn_profile_reset", "rattn_profile_count", "rattn_profile_get"]


class RattnParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("window", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float), ("rms_eps", ctypes.c_float),
                ("save_for_bwd", ctypes.c_int32), ("feature_map", ctypes.c_int32), ("kernel_path", ctypes.c_int32),
                ("state_policy", ctypes.c_int32)]


class RattnDecodeParams(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
                ("window", ctypes.c_int32), ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("rms_eps", ctypes.c_float), ("feature_map", ctypes.c_int32)]


class RattnError(RuntimeError):
    def __init__(self, status, detail):
        super().__init__(f"librattn status {status}: {detail}")
        self.status = status
        self.detail = detail


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2506_15545_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    L.rattn_workspace_bytes.restype = ctypes.c_int
    L.rattn_workspace_bytes.argtypes = [ctypes.POINTER(RattnParams)] + [ctypes.POINTER(sz)] * 3
    L.rattn_fwd.restype = ctypes.c_int
    L.rattn_fwd.argtypes = [ctypes.POINTER(RattnParams)] + [vp] * 8 + [sz, vp]
    L.rattn_fwd_static.restype = ctypes.c_int
    L.rattn_fwd_static.argtypes = [ctypes.POINTER(RattnParams)] + [vp] * 8
    L.rattn_bwd.restype = ctypes.c_int
    L.rattn_bwd.argtypes = [ctypes.POINTER(RattnParams)] + [vp] * 13 + [sz, vp]
    L.rattn_decode_step.restype = ctypes.c_int
    L.rattn_decode_step.argtypes = [ctypes.POINTER(RattnDecodeParams)] + [vp] * 11
    L.rattn_prefill_export_workspace_bytes.restype = ctypes.c_int
    L.rattn_prefill_export_workspace_bytes.argtypes = [ctypes.POINTER(RattnParams), ctypes.POINTER(sz)]
    L.rattn_prefill_export.restype = ctypes.c_int
    L.rattn_prefill_export.argtypes = [ctypes.POINTER(RattnParams)] + [vp] * 6 + [sz, vp]
    L.rattn_prefill_chunk_workspace_bytes.restype = ctypes.c_int
    L.rattn_prefill_chunk_workspace_bytes.argtypes = [ctypes.POINTER(RattnParams), ctypes.c_int32, ctypes.POINTER(sz)]
    L.rattn_prefill_chunk.restype = ctypes.c_int
    L.rattn_prefill_chunk.argtypes = [ctypes.POINTER(RattnParams), ctypes.c_int32] + [vp] * 10 + [sz, vp]
    L.rattn_cache_bytes.restype = ctypes.c_int
    L.rattn_cache_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                    ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double)]
    L.rattn_step_time_model.restype = ctypes.c_int
    L.rattn_step_time_model.argtypes = [ctypes.c_double] * 6 + [ctypes.POINTER(ctypes.c_double)]
    L.rattn_probe_mfma.restype = ctypes.c_int
    L.rattn_probe_mfma.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), vp]
    L.rattn_status_string.restype = ctypes.c_char_p
    L.rattn_status_string.argtypes = [ctypes.c_int]
    L.rattn_last_error.restype = ctypes.c_char_p
    L.rattn_version.restype = ctypes.c_char_p
    L.rattn_profile_enable.restype = None
    L.rattn_profile_enable.argtypes = [ctypes.c_int]
    L.rattn_profile_reset.restype = None
    L.rattn_profile_count.restype = ctypes.c_int
    L.rattn_profile_get.restype = ctypes.c_int
    L.rattn_profile_get.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float)]
    _lib = L
    return L


def _check(status):
    if status != 0:
        raise RattnError(status, lib().rattn_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_params(q, k, window, chunk=0, softmax_scale=1.0, rms_eps=1e-6, save_for_bwd=False, feature_map="softmax",
                kernel_path="auto", state_policy="keep"):
    B, T, Hq, D = q.shape
    return RattnParams(B, T, Hq, k.shape[2], D, window, chunk, _DTYPES[q.dtype], softmax_scale, rms_eps,
                       1 if save_for_bwd else 0, FEATURE_MAPS[feature_map], KERNEL_PATHS[kernel_path],
                       STATE_POLICIES[state_policy])


def rattn_workspace_bytes(params):
    """(fwd_bytes, bwd_bytes, saved_bytes) for a RattnParams."""
    f, b, s = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().rattn_workspace_bytes(ctypes.byref(params), ctypes.byref(f), ctypes.byref(b), ctypes.byref(s)))
    return f.value, b.value, s.value


def _check_layer(q, k, v):
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not (t.is_cuda and t.is_contiguous() and t.dim() == 4):
            raise ValueError(f"{name} must be a contiguous 4-d device tensor [B,T,H,D]")
    if k.shape != v.shape or k.shape[0] != q.shape[0] or k.shape[1] != q.shape[1] or k.shape[3] != q.shape[3]:
        raise ValueError("q/k/v shapes do not match")
    if q.dtype not in _DTYPES or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share dtype float32 or bfloat16")


def _gain(g, Hq, D, dev):
    if g is None:
        return None
    g = g.to(device=dev, dtype=torch.float32).contiguous()
    if g.shape != (Hq, D):
        raise ValueError("gains must be [Hq, D]")
    return g


def _bytes(n, dev):
    return torch.empty(max(int(n), 16), dtype=torch.uint8, device=dev)


def rattn_fwd(q, k, v, window, gamma_swa=None, gamma_rla=None, chunk=0, softmax_scale=1.0, rms_eps=1e-6,
              save_for_bwd=False, out=None, saved=None, workspace=None, feature_map="softmax", kernel_path="auto",
              state_policy="keep"):
    """o = RMS(SWA(q,k,v)) + RMS(RLA(q,k,v)); returns o, or (o, saved) when save_for_bwd.

    out / saved / workspace may be passed in to reuse buffers (uint8 tensors for the latter two)."""
    _check_layer(q, k, v)
    p = make_params(q, k, window, chunk, softmax_scale, rms_eps, save_for_bwd, feature_map, kernel_path, state_policy)
    fwd_b, _, saved_b = rattn_workspace_bytes(p)
    dev = q.device
    o = torch.empty_like(q) if out is None else out
    ws = _bytes(fwd_b, dev) if workspace is None else workspace
    sv = None
    if save_for_bwd:
        sv = _bytes(saved_b, dev) if saved is None else saved
    gs = _gain(gamma_swa, q.shape[2], q.shape[3], dev)
    gr = _gain(gamma_rla, q.shape[2], q.shape[3], dev)
    _check(lib().rattn_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(gs), _ptr(gr), _ptr(o), _ptr(sv),
                           _ptr(ws), ws.numel(), _stream()))
    return (o, sv) if save_for_bwd else o


STATIC_SCRATCH_BYTES = 96 << 20


def rattn_fwd_static(q, k, v, window, out, gamma_swa=None, gamma_rla=None, chunk=0, softmax_scale=1.0, rms_eps=1e-6,
                     saved=None, feature_map="softmax"):
    """rattn_fwd on the library's built-in scratch buffer: nothing is allocated here or in the library.  `out`
    (and `saved`, which switches save_for_bwd on) are the caller's tensors; gains must already be fp32 [Hq,D] device
    tensors.  Returns out."""
    _check_layer(q, k, v)
    for g in (gamma_swa, gamma_rla):
        if g is not None and not (g.is_cuda and g.is_contiguous() and g.dtype == torch.float32
                                  and tuple(g.shape) == (q.shape[2], q.shape[3])):
            raise ValueError("gains must be contiguous fp32 [Hq, D] device tensors")
    if out.shape != q.shape or out.dtype != q.dtype or not (out.is_cuda and out.is_contiguous()):
        raise ValueError("out must match q")
    p = make_params(q, k, window, chunk, softmax_scale, rms_eps, saved is not None, feature_map)
    _check(lib().rattn_fwd_static(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(gamma_swa), _ptr(gamma_rla),
                                  _ptr(out), _ptr(saved), _stream()))
    return out


def rattn_bwd(q, k, v, saved, dO, window, gamma_swa=None, gamma_rla=None, chunk=0, softmax_scale=1.0,
              rms_eps=1e-6, want_dgamma=True, workspace=None, out=None, feature_map="softmax", kernel_path="auto",
              state_policy="keep"):
    """(dq, dk, dv, dgamma_swa, dgamma_rla) for upstream gradient dO; `saved` from rattn_fwd (same kernel_path)."""
    _check_layer(q, k, v)
    if dO.shape != q.shape or dO.dtype != q.dtype or not dO.is_contiguous():
        raise ValueError("dO must match q")
    p = make_params(q, k, window, chunk, softmax_scale, rms_eps, True, feature_map, kernel_path, state_policy)
    _, bwd_b, saved_b = rattn_workspace_bytes(p)
    if saved is None or saved.numel() < saved_b:
        raise ValueError("saved buffer missing or too small")
    dev = q.device
    ws = _bytes(bwd_b, dev) if workspace is None else workspace
    if out is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    else:
        dq, dk, dv = out
    dgs = dgr = None
    if want_dgamma:
        dgs = torch.empty(q.shape[2], q.shape[3], dtype=torch.float32, device=dev)
        dgr = torch.empty_like(dgs)
    gs = _gain(gamma_swa, q.shape[2], q.shape[3], dev)
    gr = _gain(gamma_rla, q.shape[2], q.shape[3], dev)
    _check(lib().rattn_bwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(gs), _ptr(gr), _ptr(saved), _ptr(dO),
                           _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dgs), _ptr(dgr), _ptr(ws), ws.numel(), _stream()))
    return dq, dk, dv, dgs, dgr


def rattn_decode_step(q, k_new, v_new, pos, k_ring, v_ring, state, gamma_swa=None, gamma_rla=None,
                      softmax_scale=1.0, rms_eps=1e-6, out=None, feature_map="softmax"):
    """One decode step; k_ring, v_ring, state are updated in place; returns o [N,Hq,D]."""
    N, Hq, D = q.shape
    Hkv, W = k_ring.shape[1], k_ring.shape[2]
    for name, t in (("q", q), ("k_new", k_new), ("v_new", v_new), ("k_ring", k_ring), ("v_ring", v_ring),
                    ("state", state), ("pos", pos)):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError(f"{name} must be a contiguous device tensor")
    if k_new.shape != (N, Hkv, D) or v_new.shape != (N, Hkv, D) or k_ring.shape != (N, Hkv, W, D) \
            or v_ring.shape != k_ring.shape or state.shape != (N, Hkv, D, D) or pos.shape != (N,):
        raise ValueError("decode tensor shapes do not match")
    if state.dtype != torch.float32 or pos.dtype != torch.int32:
        raise ValueError("state must be float32 and pos int32")
    if q.dtype not in _DTYPES or any(t.dtype != q.dtype for t in (k_new, v_new, k_ring, v_ring)):
        raise ValueError("q, k_new, v_new and the rings must share dtype float32 or bfloat16")
    p = RattnDecodeParams(N, Hq, Hkv, D, W, _DTYPES[q.dtype], softmax_scale, rms_eps, FEATURE_MAPS[feature_map])
    o = torch.empty_like(q) if out is None else out
    gs = _gain(gamma_swa, Hq, D, q.device)
    gr = _gain(gamma_rla, Hq, D, q.device)
    _check(lib().rattn_decode_step(ctypes.byref(p), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(pos), _ptr(k_ring),
                                   _ptr(v_ring), _ptr(state), _ptr(gs), _ptr(gr), _ptr(o), _stream()))
    return o


def rattn_prefill_export(k, v, window, k_ring=None, v_ring=None, state=None, feature_map="softmax"):
    """Rings and lagged state a decode step at pos = T expects after the prompt k, v [B,T,Hkv,D].
    Returns (k_ring [B,Hkv,W,D], v_ring, state [B,Hkv,D,D] fp32); ring slots the prompt does not reach are zero
    when the rings are allocated here."""
    B, T, Hkv, D = k.shape
    for name, t in (("k", k), ("v", v)):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError(f"{name} must be a contiguous device tensor")
    if v.shape != k.shape or v.dtype != k.dtype or k.dtype not in _DTYPES:
        raise ValueError("k and v must share shape and dtype float32 or bfloat16")
    p = RattnParams(B, T, Hkv, Hkv, D, window, 0, _DTYPES[k.dtype], 1.0, 1e-6, 0, FEATURE_MAPS[feature_map], 0, 0)
    if k_ring is None:
        k_ring = torch.zeros(B, Hkv, window, D, dtype=k.dtype, device=k.device)
    if v_ring is None:
        v_ring = torch.zeros(B, Hkv, window, D, dtype=k.dtype, device=k.device)
    if state is None:
        state = torch.empty(B, Hkv, D, D, dtype=torch.float32, device=k.device)
    nbytes = ctypes.c_size_t()
    _check(lib().rattn_prefill_export_workspace_bytes(ctypes.byref(p), ctypes.byref(nbytes)))
    ws = torch.empty(max(nbytes.value, 16), dtype=torch.uint8, device=k.device)
    _check(lib().rattn_prefill_export(ctypes.byref(p), _ptr(k), _ptr(v), _ptr(k_ring), _ptr(v_ring), _ptr(state),
                                      _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return k_ring, v_ring, state


def rattn_prefill_chunk(q, k, v, window, pos0, k_ring, v_ring, state, gamma_swa=None, gamma_rla=None, chunk=0,
                        softmax_scale=1.0, rms_eps=1e-6, workspace=None, out=None, feature_map="softmax"):
    """Layer output for tokens pos0 .. pos0+T-1 (q [B,T,Hq,D], k, v [B,T,Hkv,D]) of sequences whose first pos0
    tokens live in k_ring, v_ring [B,Hkv,W,D] and state [B,Hkv,D,D] fp32; those three are updated in place to
    position pos0 + T.  Returns o [B,T,Hq,D]."""
    _check_layer(q, k, v)
    for name, t in (("k_ring", k_ring), ("v_ring", v_ring), ("state", state)):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError(f"{name} must be a contiguous device tensor")
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]
    if tuple(k_ring.shape) != (B, Hkv, window, D) or v_ring.shape != k_ring.shape or k_ring.dtype != q.dtype or \
            v_ring.dtype != q.dtype:
        raise ValueError("k_ring, v_ring must be [B,Hkv,window,D] in the dtype of q")
    if tuple(state.shape) != (B, Hkv, D, D) or state.dtype != torch.float32:
        raise ValueError("state must be fp32 [B,Hkv,D,D]")
    p = make_params(q, k, window, chunk, softmax_scale, rms_eps, False, feature_map)
    nbytes = ctypes.c_size_t()
    _check(lib().rattn_prefill_chunk_workspace_bytes(ctypes.byref(p), int(pos0), ctypes.byref(nbytes)))
    if workspace is None:
        workspace = torch.empty(max(nbytes.value, 16), dtype=torch.uint8, device=q.device)
    elif not (workspace.is_cuda and workspace.is_contiguous() and workspace.dtype == torch.uint8):
        raise ValueError("workspace must be a contiguous uint8 device tensor")
    o = torch.empty_like(q) if out is None else out
    gs = _gain(gamma_swa, Hq, D, q.device)   # fp32 [Hq,D] on the device, kept alive until the call has been enqueued
    gr = _gain(gamma_rla, Hq, D, q.device)
    _check(lib().rattn_prefill_chunk(ctypes.byref(p), int(pos0), _ptr(q), _ptr(k), _ptr(v), _ptr(gs),
                                     _ptr(gr), _ptr(k_ring), _ptr(v_ring), _ptr(state), _ptr(o), _ptr(workspace),
                                     ctypes.c_size_t(workspace.numel()), _stream()))
    return o


def rattn_cache_bytes(layers, global_every, ctx, window, with_state, Hkv, D, elem_bytes):
    """Decode-cache bytes of one sequence in a local-global stack (host arithmetic, nothing is launched)."""
    out = ctypes.c_double()
    _check(lib().rattn_cache_bytes(layers, global_every, ctx, window, 1 if with_state else 0, Hkv, D, elem_bytes,
                                   ctypes.byref(out)))
    return out.value


def rattn_step_time_model(batch, cache_bytes, param_count, param_bytes, bandwidth, flops):
    """Theoretical generation step time in seconds (host arithmetic, nothing is launched)."""
    out = ctypes.c_double()
    _check(lib().rattn_step_time_model(batch, cache_bytes, param_count, param_bytes, bandwidth, flops, ctypes.byref(out)))
    return out.value


def rattn_probe_mfma(sink, iters, blocks):
    """Enqueue the matrix-core probe loop on the current stream; returns the FLOPs it issues."""
    flops = ctypes.c_double()
    _check(lib().rattn_probe_mfma(_ptr(sink), iters, blocks, ctypes.byref(flops), _stream()))
    return flops.value


def rattn_profile_enable(on):
    lib().rattn_profile_enable(1 if on else 0)


def rattn_profile_reset():
    lib().rattn_profile_reset()


def rattn_profile_records():
    """[(kernel name, milliseconds)] of every launch since the last reset (waits for them)."""
    L = lib()
    out = []
    for i in range(L.rattn_profile_count()):
        name, ms = ctypes.c_char_p(), ctypes.c_float()
        _check(L.rattn_profile_get(i, ctypes.byref(name), ctypes.byref(ms)))
        out.append((name.value.decode(), ms.value))
    return out
