"""fp64 CPU oracle for the RAttention layer (sliding-window attention + residual linear attention).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module: it is
used by tests/, by the smoke check and by the cpu_baseline leg of the benchmark.  It
shares no code with the HIP kernels and is deliberately plain and slow.

Conventions
-----------
* Tensors are numpy float64 arrays laid out [B, T, H, D] (q has Hq heads, k/v have Hkv).
* Positions are 0-based here.  `W` is the number of keys the softmax branch sees,
  *including* the current token: the window of query t is {s : max(0, t-W+1) <= s <= t}
  and the residual (out-of-window) set is {s : 0 <= s <= t-W}.  The paper writes the
  same partition with w = W-1 (Sec. 2.1 SWA sum from t-w to t; Eq. 4 reads S_{t-w-1}).
* Query head h uses KV head h // (Hq // Hkv)  (Sec. 3.1, group-query variant).
* phi = softmax over the feature axis (Sec. 3.1 "Parameterization", Sec. 4.5 ablation);
  the paper prints no formula for phi, so this reading is "parity unpinned" by the paper.
  The ablation's two alternatives are selectable with feature_map="relu" (max(x, 0) per
  feature) and feature_map="identity" (phi(x) = x); every function takes the argument.
* RMS epsilon and gains [H, D] per branch (Sec. 3.2) are arguments; the paper gives no
  defaults ("parity unpinned" for eps / gain shape).

Every function cites the passage it follows.  Pins live in tests/test_oracle_*.py.
"""
import numpy as np


# ----------------------------------------------------------------------------- index sets
def window_set_1based(t, W):
    """Keys (1-based) seen by the softmax branch for 1-based query t.  Sec. 2.1 (SWA)."""
    return list(range(max(1, t - W + 1), t + 1))


def residual_set_1based(t, W):
    """Keys (1-based) summarised by the linear branch for 1-based query t.  Eq. 4 / Fig. 1."""
    return list(range(1, t - W + 1))


# ----------------------------------------------------------------------------- pieces
FEATURE_MAPS = ("softmax", "relu", "identity")


def phi(x, feature_map="softmax"):
    """Feature map over the last (feature) axis.  Sec. 3.1: softmax (the layer's choice);
    Sec. 4.5 ablation: ReLU and identity."""
    x = np.asarray(x, dtype=np.float64)
    if feature_map == "softmax":
        m = np.max(x, axis=-1, keepdims=True)
        e = np.exp(x - m)
        return e / np.sum(e, axis=-1, keepdims=True)
    if feature_map == "relu":
        return np.maximum(x, 0.0)
    if feature_map == "identity":
        return x.copy()
    raise ValueError(f"unknown feature map {feature_map!r}")


def phi_bwd(x, f, df, feature_map="softmax"):
    """Gradient with respect to x of sum(phi(x) * df), f = phi(x), rows on the last axis.
    softmax: f*(df - <df, f>);  ReLU: df where x > 0 (0 at x = 0);  identity: df."""
    if feature_map == "softmax":
        return f * (df - np.sum(df * f, axis=-1, keepdims=True))
    if feature_map == "relu":
        return np.where(np.asarray(x) > 0.0, df, 0.0)
    if feature_map == "identity":
        return np.array(df, dtype=np.float64)
    raise ValueError(f"unknown feature map {feature_map!r}")


def rms(x, gamma, eps):
    """gamma * x / sqrt(mean(x^2) + eps) over the last axis; returns (y, rstd).  Sec. 3.2."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return gamma * x * r, r[..., 0]


def _gains(g, H, D):
    if g is None:
        return np.ones((H, D), dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    assert g.shape == (H, D)
    return g


# ----------------------------------------------------------------------------- O1: explicit loops
def fwd_loops(q, k, v, W, scale=1.0, eps=1e-6, gamma_swa=None, gamma_rla=None, feature_map="softmax"):
    """The layer written out token by token (tiny inputs only).

    softmax branch: Sec. 2.1 SWA formula;  linear branch: Eq. 4 unrolled with
    S_t = sum_i phi(k_i)^T v_i (Sec. 2.2), no normaliser (Eq. 1);  combination: Sec. 3.2.
    Returns dict(o, xs, xr).
    """
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    gs = _gains(gamma_swa, Hq, D); gr = _gains(gamma_rla, Hq, D)
    o = np.zeros_like(q); xs = np.zeros_like(q); xr = np.zeros_like(q)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for t in range(T):
                qt = q[b, t, h]
                # softmax over the window
                win = range(max(0, t - W + 1), t + 1) if W > 0 else range(0)
                if len(win) > 0:
                    logits = np.array([scale * np.dot(qt, k[b, s, g]) for s in win])
                    e = np.exp(logits - logits.max())
                    num = np.zeros(D)
                    for wgt, s in zip(e, win):
                        num += wgt * v[b, s, g]
                    xs[b, t, h] = num / e.sum()
                # explicit sum over the out-of-window tokens
                qf = phi(qt, feature_map)
                acc = np.zeros(D)
                for s in range(0, t - W + 1):
                    acc += np.dot(qf, phi(k[b, s, g], feature_map)) * v[b, s, g]
                xr[b, t, h] = acc
                ys, _ = rms(xs[b, t, h], gs[h], eps)
                yr, _ = rms(xr[b, t, h], gr[h], eps)
                o[b, t, h] = ys + yr
    return dict(o=o, xs=xs, xr=xr)


# ----------------------------------------------------------------------------- O2: dense masked form
def _masks(rows, T, W):
    t = np.asarray(rows)[:, None]
    s = np.arange(T)[None, :]
    win = (s <= t) & (s > t - W)
    res = s <= t - W
    return win, res


def fwd_dense(q, k, v, W, scale=1.0, eps=1e-6, gamma_swa=None, gamma_rla=None,
              rows=None, heads=None, batches=None, row_block=1024, feature_map="softmax"):
    """Same definition as fwd_loops, with the sums over keys written as masked matrix
    products per head (rows of queries are independent, so they are taken in batches).

    rows / heads / batches restrict which outputs are computed (others stay 0).
    Returns dict(o, xs, xr, lse, rs, rr); lse/rs/rr are [B, Hq, T].
    """
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    gs = _gains(gamma_swa, Hq, D); gr = _gains(gamma_rla, Hq, D)
    rows = np.arange(T) if rows is None else np.asarray(rows)
    heads = range(Hq) if heads is None else heads
    batches = range(B) if batches is None else batches
    o = np.zeros_like(q); xs = np.zeros_like(q); xr = np.zeros_like(q)
    lse = np.zeros((B, Hq, T)); rs = np.zeros((B, Hq, T)); rr = np.zeros((B, Hq, T))
    for b in batches:
        for h in heads:
            g = h // G
            kk = k[b, :, g]; vv = v[b, :, g]
            kf = phi(kk, feature_map)
            for r0 in range(0, len(rows), row_block):
                rr_ = rows[r0:r0 + row_block]
                win, res = _masks(rr_, T, W)
                qq = q[b, rr_, h]
                a = scale * (qq @ kk.T)
                a = np.where(win, a, -np.inf)
                if W > 0:
                    m = a.max(axis=1, keepdims=True)
                    e = np.exp(a - m)
                    z = e.sum(axis=1, keepdims=True)
                    x_s = (e / z) @ vv
                    lse[b, h, rr_] = (m + np.log(z))[:, 0]
                else:
                    x_s = np.zeros((len(rr_), D))
                c = np.where(res, phi(qq, feature_map) @ kf.T, 0.0)
                x_r = c @ vv
                ys, r_s = rms(x_s, gs[h], eps)
                yr, r_r = rms(x_r, gr[h], eps)
                xs[b, rr_, h] = x_s; xr[b, rr_, h] = x_r
                rs[b, h, rr_] = r_s; rr[b, h, rr_] = r_r
                o[b, rr_, h] = ys + yr
    return dict(o=o, xs=xs, xr=xr, lse=lse, rs=rs, rr=rr)


# ----------------------------------------------------------------------------- linear branch, other forms
def rla_recurrent(q, k, v, W, feature_map="softmax"):
    """Eq. 4 as a recurrence: S_t = S_{t-1} + phi(k_t)^T v_t, readout phi(q_t) S_{t-W}
    (0-based: state that has absorbed keys 0..t-W).  S before any key is 0 (Sec. 2.2)."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]; G = Hq // Hkv
    out = np.zeros_like(q)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            S = np.zeros((D, D))
            for t in range(T):
                if t - W >= 0:
                    S = S + np.outer(phi(k[b, t - W, g], feature_map), v[b, t - W, g])
                out[b, t, h] = phi(q[b, t, h], feature_map) @ S
    return out


def rla_chunkwise(q, k, v, W, C, feature_map="softmax"):
    """Eqs. 2-3 at lag W.  Key chunk j holds keys jC..(j+1)C-1; S_[j] is the sum over
    chunks before j; the query paired with key position p = t-W sits in chunk p // C and
    adds the intra-chunk masked product with M[t', s'] = 1 if s' <= t' (diagonal kept,
    because Eq. 1 reads a state that already holds the current key)."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]; G = Hq // Hkv
    out = np.zeros_like(q)
    Tp = T - W
    if Tp <= 0:
        return out
    nch = (Tp + C - 1) // C
    M = np.tril(np.ones((C, C)))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            S = np.zeros((D, D))
            for j in range(nch):
                lo, hi = j * C, min((j + 1) * C, Tp)
                n = hi - lo
                Qt = phi(q[b, lo + W:hi + W, h], feature_map)
                Kt = phi(k[b, lo:hi, g], feature_map); V = v[b, lo:hi, g]
                out[b, lo + W:hi + W, h] = Qt @ S + ((Qt @ Kt.T) * M[:n, :n]) @ V
                S = S + Kt.T @ V
    return out


def linear_attention_eq1(q, k, v, feature_map="softmax"):
    """Eq. 1: o_t = phi(q_t) S_t with S_t the running sum of phi(k)^T v (current token
    included), written with a cumulative sum of outer products.  Single head [T, D]."""
    kf = phi(k, feature_map); qf = phi(q, feature_map)
    S = np.cumsum(kf[:, :, None] * np.asarray(v, np.float64)[:, None, :], axis=0)
    return np.einsum('tf,tfd->td', qf, S)


# ----------------------------------------------------------------------------- backward
def bwd_dense(q, k, v, dO, W, scale=1.0, eps=1e-6, gamma_swa=None, gamma_rla=None,
              heads=None, batches=None, rows=None, row_block=1024, feature_map="softmax"):
    """Analytic gradient of sum(o * dO) for the layer of fwd_dense.

    Epilogue (Sec. 3.2): y = g*x*r, r = (mean x^2 + eps)^-1/2  =>
        dx = r*(g*dy) - x * r^3 * mean(g*dy*x),   dgamma += dy * x * r.
    Softmax branch (Sec. 2.1): dv_s += p dx,  dp = <dx, v_s>,  da = p (dp - sum p dp),
        dq += scale*da k_s,  dk_s += scale*da q_t.
    Linear branch (Eq. 4 unrolled): dv_s += c dx, dc = <dx, v_s>, dphi(q) += dc phi(k_s),
        dphi(k_s) += dc phi(q); then through phi (phi_bwd; for softmax dx_in = f*(df - <df, f>)).
    `rows` restricts the set of query rows whose contributions are included (dq of other
    rows stays 0; dk/dv then hold only the contributions of those rows).
    Returns dict(dq, dk, dv, dgamma_swa, dgamma_rla).
    """
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    dO = np.asarray(dO, np.float64)
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]; G = Hq // Hkv
    gs = _gains(gamma_swa, Hq, D); gr = _gains(gamma_rla, Hq, D)
    rows = np.arange(T) if rows is None else np.asarray(rows)
    heads = range(Hq) if heads is None else heads
    batches = range(B) if batches is None else batches
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    dgs = np.zeros((Hq, D)); dgr = np.zeros((Hq, D))
    for b in batches:
        for h in heads:
            g = h // G
            kk = k[b, :, g]; vv = v[b, :, g]
            kf = phi(kk, feature_map)
            dkf = np.zeros((T, D))
            for r0 in range(0, len(rows), row_block):
                rr_ = rows[r0:r0 + row_block]
                win, res = _masks(rr_, T, W)
                qq = q[b, rr_, h]; dy = dO[b, rr_, h]
                qf = phi(qq, feature_map)
                # forward pieces
                if W > 0:
                    a = np.where(win, scale * (qq @ kk.T), -np.inf)
                    e = np.exp(a - a.max(axis=1, keepdims=True))
                    p = e / e.sum(axis=1, keepdims=True)
                    x_s = p @ vv
                else:
                    p = np.zeros((len(rr_), T)); x_s = np.zeros((len(rr_), D))
                c = np.where(res, qf @ kf.T, 0.0)
                x_r = c @ vv
                # epilogue backward
                def rms_bwd(x, gam):
                    r = 1.0 / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + eps)
                    gy = gam[None, :] * dy
                    dx = r * gy - x * (r ** 3) * np.mean(gy * x, axis=1, keepdims=True)
                    return dx, (dy * x * r).sum(axis=0)
                dxs, dg1 = rms_bwd(x_s, gs[h]); dgs[h] += dg1
                dxr, dg2 = rms_bwd(x_r, gr[h]); dgr[h] += dg2
                # softmax branch
                dv[b, :, g] += p.T @ dxs
                dp = dxs @ vv.T
                da = p * (dp - np.sum(p * dp, axis=1, keepdims=True))
                dq[b, rr_, h] += scale * (da @ kk)
                dk[b, :, g] += scale * (da.T @ qq)
                # linear branch
                dv[b, :, g] += c.T @ dxr
                dc = np.where(res, dxr @ vv.T, 0.0)
                dqf = dc @ kf
                dkf += dc.T @ qf
                dq[b, rr_, h] += phi_bwd(qq, qf, dqf, feature_map)
            dk[b, :, g] += phi_bwd(kk, kf, dkf, feature_map)
    return dict(dq=dq, dk=dk, dv=dv, dgamma_swa=dgs, dgamma_rla=dgr)


# ----------------------------------------------------------------------------- decode
def decode_step(q, k_new, v_new, pos, k_ring, v_ring, state, W, scale=1.0, eps=1e-6,
                gamma_swa=None, gamma_rla=None, feature_map="softmax"):
    """One generated token per sequence with constant memory (Sec. 2.1 window cache of the
    last W keys, Sec. 2.2 fixed-size state; the paper leaves the procedure to the reader).

    q [N,Hq,D]; k_new, v_new [N,Hkv,D]; pos [N] 0-based index of the new token;
    k_ring, v_ring [N,Hkv,W,D] hold key s in slot s % W; state [N,Hkv,D,D] (rows = feature,
    cols = value) holds, before the call, the sum of phi(k_s)^T v_s over s <= pos-1-W (what
    the previous token's query read).
    Step: the key leaving the window (index pos-W, stored in slot pos % W) is folded into
    the state, the slot is overwritten with the new key/value, then the softmax branch reads
    min(pos+1, W) slots and the linear branch reads phi(q) S_{pos-W}.
    Returns (o [N,Hq,D], k_ring', v_ring', state') as new arrays.
    """
    q = np.asarray(q, np.float64)
    k_ring = np.array(k_ring, np.float64); v_ring = np.array(v_ring, np.float64)
    state = np.array(state, np.float64)
    N, Hq, D = q.shape
    Hkv = k_new.shape[1]; G = Hq // Hkv
    gs = _gains(gamma_swa, Hq, D); gr = _gains(gamma_rla, Hq, D)
    o = np.zeros((N, Hq, D))
    for n in range(N):
        p = int(pos[n]); slot = p % W
        for g in range(Hkv):
            if p >= W:
                state[n, g] += np.outer(phi(k_ring[n, g, slot], feature_map), v_ring[n, g, slot])
            k_ring[n, g, slot] = k_new[n, g]; v_ring[n, g, slot] = v_new[n, g]
            nvalid = min(p + 1, W)
            for hh in range(G):
                h = g * G + hh
                a = scale * (k_ring[n, g, :nvalid] @ q[n, h])
                e = np.exp(a - a.max())
                x_s = (e / e.sum()) @ v_ring[n, g, :nvalid]
                x_r = phi(q[n, h], feature_map) @ state[n, g]
                ys, _ = rms(x_s, gs[h], eps); yr, _ = rms(x_r, gr[h], eps)
                o[n, h] = ys + yr
    return o, k_ring, v_ring, state


def prefill_export(k, v, W, feature_map="softmax"):
    """What a decode step at pos = T expects after a prompt of T tokens (the hand-over the paper's
    inference discussion implies, Sec. 2.1 / 2.2 / 4.4): rings with key/value s in slot s % W for the last
    min(T, W) tokens (other slots zero), and the state sum_{s < T-W} phi(k_s)^T v_s (rows = feature,
    columns = value), i.e. the S_{t-W} that Eq. 4 lets query t = T read.
    k, v [B,T,Hkv,D]; returns (k_ring [B,Hkv,W,D], v_ring, state [B,Hkv,D,D])."""
    k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    B, T, Hkv, D = k.shape
    k_ring = np.zeros((B, Hkv, W, D)); v_ring = np.zeros((B, Hkv, W, D))
    state = np.zeros((B, Hkv, D, D))
    for b in range(B):
        for g in range(Hkv):
            for s in range(max(0, T - W), T):
                k_ring[b, g, s % W] = k[b, s, g]; v_ring[b, g, s % W] = v[b, s, g]
            for s in range(0, T - W):
                state[b, g] += np.outer(phi(k[b, s, g], feature_map), v[b, s, g])
    return k_ring, v_ring, state


# ----------------------------------------------------------------------------- closed forms in the text
def kv_cache_saving(layers, global_every, ctx, w_from, w_to):
    """Fraction of KV cache saved when local layers shrink their window (Sec. 1 example):
    one global layer in every `global_every` layers keeps min(ctx, ctx), local ones min(ctx, w)."""
    n_glob = layers // global_every
    n_loc = layers - n_glob
    before = n_glob * ctx + n_loc * min(ctx, w_from)
    after = n_glob * ctx + n_loc * min(ctx, w_to)
    return 1.0 - after / before


def state_equivalent_window(d_feat, d):
    """Window size whose KV cache equals one d' x d state (Sec. 2.2 and its footnote)."""
    return d_feat * d / (2 * d)


def decode_step_time(batch, kv_bytes_per_seq, param_count, param_bytes, bw, flops):
    """Theoretical generation step time (Sec. 4.4):
    B*S_KV/BW + max(2*B*P_count/F, P_size/BW)."""
    return batch * kv_bytes_per_seq / bw + max(2.0 * batch * param_count / flops, param_bytes / bw)
