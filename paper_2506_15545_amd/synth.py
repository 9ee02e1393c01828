"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds none of the method's arithmetic: only random draws, casts and shapes.
The workloads follow the paper's pretraining layers (Table 1: head size 128, GQA;
Sec. 4.3: context 4096 / 8192, window 512) with the head counts of the benchmark
configurations; the paper's own data is a private web crawl, so i.i.d. normal
q/k/v stand in for it.
"""
from dataclasses import dataclass
import math
import torch


@dataclass(frozen=True)
class LayerConfig:
    name: str
    B: int
    T: int
    Hq: int
    Hkv: int
    D: int
    W: int
    chunk: int
    dtype: str          # "f32" | "bf16"
    seed: int
    input_std: float    # std of q, k, v entries
    scale: float        # softmax_scale of the softmax branch


CONFIGS = {
    # tiny fp32 forward: inputs pre-scaled by 1/sqrt(64), paper formula verbatim (scale 1)
    "tiny_f32": LayerConfig("tiny_f32", 1, 256, 2, 2, 64, 32, 16, "f32", 0, 1.0 / 8.0, 1.0),
    # 3B-scale layer
    "layer3b_t4096_w512": LayerConfig("layer3b_t4096_w512", 4, 4096, 24, 8, 128, 512, 64, "bf16", 1,
                                      1.0, 1.0 / math.sqrt(128.0)),
    # 12B-scale layer
    "layer12b_t8192_w512": LayerConfig("layer12b_t8192_w512", 2, 8192, 32, 8, 128, 512, 64, "bf16", 2,
                                       1.0, 1.0 / math.sqrt(128.0)),
}


def sweep_config(W):
    """Window sweep at T=8192 (W in {128, 512, 1024, 4096, 8192}; W=T is the causal case)."""
    return LayerConfig(f"sweep_t8192_w{W}", 4, 8192, 24, 8, 128, W, 64, "bf16", 3,
                       1.0, 1.0 / math.sqrt(128.0))


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_layer_inputs(cfg, with_dO=False, B=None, T=None):
    """q [B,T,Hq,D], k, v [B,T,Hkv,D] (and dO) on the CPU in cfg.dtype.

    Draw order is q, k, v, (dO) from one generator seeded with cfg.seed, fp32 normal
    times input_std, then one cast to the I/O dtype.  B/T may be overridden to cut a
    cheaper case of the same recipe.
    """
    B = cfg.B if B is None else B
    T = cfg.T if T is None else T
    g = torch.Generator().manual_seed(cfg.seed)
    dt = torch_dtype(cfg.dtype)
    q = (torch.randn(B, T, cfg.Hq, cfg.D, generator=g) * cfg.input_std).to(dt)
    k = (torch.randn(B, T, cfg.Hkv, cfg.D, generator=g) * cfg.input_std).to(dt)
    v = (torch.randn(B, T, cfg.Hkv, cfg.D, generator=g) * cfg.input_std).to(dt)
    out = [q, k, v]
    if with_dO:
        out.append(torch.randn(B, T, cfg.Hq, cfg.D, generator=g).to(dt))
    return out


def make_random_layer(B, T, Hq, Hkv, D, dtype, seed, std=1.0, with_dO=False, with_gains=False):
    """Free-form variant of make_layer_inputs for parity cases of arbitrary shape."""
    g = torch.Generator().manual_seed(seed)
    dt = torch_dtype(dtype)
    q = (torch.randn(B, T, Hq, D, generator=g) * std).to(dt)
    k = (torch.randn(B, T, Hkv, D, generator=g) * std).to(dt)
    v = (torch.randn(B, T, Hkv, D, generator=g) * std).to(dt)
    out = {"q": q, "k": k, "v": v}
    if with_dO:
        out["dO"] = torch.randn(B, T, Hq, D, generator=g).to(dt)
    if with_gains:
        out["gamma_swa"] = 1.0 + 0.25 * torch.randn(Hq, D, generator=g)
        out["gamma_rla"] = 1.0 + 0.25 * torch.randn(Hq, D, generator=g)
    return out


@dataclass(frozen=True)
class DecodeConfig:
    name: str
    N: int              # sequences
    Hq: int
    Hkv: int
    D: int
    W: int
    dtype: str
    seed: int
    pos_lo: int
    pos_hi: int
    scale: float


DECODE_CONFIGS = {
    "decode_b128_w512": DecodeConfig("decode_b128_w512", 128, 32, 8, 128, 512, "bf16", 4, 512, 32768,
                                     1.0 / math.sqrt(128.0)),
}


def make_decode_inputs(cfg, N=None, pos=None):
    """One decode step's inputs on the CPU.

    ring and new token ~ N(0,1); pos ~ U{pos_lo..pos_hi}; state entries ~
    N(0, (pos-W) * e / D^2): the variance a sum of (pos-W) outer products of a softmax
    feature row (mean-square about e/D^2 for N(0,1) keys) with an N(0,1) value row has.
    """
    N = cfg.N if N is None else N
    g = torch.Generator().manual_seed(cfg.seed)
    dt = torch_dtype(cfg.dtype)
    q = torch.randn(N, cfg.Hq, cfg.D, generator=g).to(dt)
    k_new = torch.randn(N, cfg.Hkv, cfg.D, generator=g).to(dt)
    v_new = torch.randn(N, cfg.Hkv, cfg.D, generator=g).to(dt)
    k_ring = torch.randn(N, cfg.Hkv, cfg.W, cfg.D, generator=g).to(dt)
    v_ring = torch.randn(N, cfg.Hkv, cfg.W, cfg.D, generator=g).to(dt)
    if pos is None:
        pos = torch.randint(cfg.pos_lo, cfg.pos_hi + 1, (N,), generator=g, dtype=torch.int32)
    else:
        pos = torch.as_tensor(pos, dtype=torch.int32)
    std = torch.sqrt(torch.clamp(pos.float() - cfg.W, min=0.0) * math.e) / cfg.D
    state = torch.randn(N, cfg.Hkv, cfg.D, cfg.D, generator=g) * std.view(N, 1, 1, 1)
    return dict(q=q, k_new=k_new, v_new=v_new, pos=pos, k_ring=k_ring, v_ring=v_ring, state=state)
