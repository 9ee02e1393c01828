"""CPU error model of the matrix-core (bf16 MFMA) path: the oracle's arithmetic in float64 with a rounding to
bf16 at every place where the kernels hand a value to the matrix cores or store it as bf16, and nowhere else.

It is test infrastructure (imported by tests only) and shares nothing with the HIP sources: the list of rounding
points below is a description of the kernels' data flow, written down here so that the parity bounds of the GPU
tests can be derived on the CPU instead of being picked by hand.

Rounding points (everything else is carried in fp32 by the kernels, float64 here):
  forward   P (softmax-branch probabilities, before the product with V; the row sum uses the unrounded values);
            phi(q), phi(k) (operands of every linear-branch product); the masked intra-chunk products
            C = phi(q) phi(k)^T (operand of C V); the chunk states (fp32 prefix sum, stored as bf16 operands,
            one per 128 keys, first state at key (W_r mod 128), W_r = window rounded up to 64);
            the saved branch outputs x^s, x^r; the output o (one rounding of the fp32 sum).
  backward  dx^s, dx^r (results of the RMS-norm backward, computed from the saved bf16 x^s, x^r);
            delta = <bf16(dx^s), saved x^s>;  dS = P (dP - delta) scale;  P again as operand of dV;
            dC = (dx^r V^T) masked; C again as operand of dV; the reverse-time states
            R = sum over later query tiles and the group's heads of phi(q)^T dx^r (bf16 operands, fp32 sum,
            stored bf16 per 128 keys); the results dq, dk, dv.
The Jacobian of phi uses the fp32 (unrounded) phi of the row.
Which pairs go through a stored state and which through the masked intra-chunk product follows the kernels' tiling:
query tile t0 = 128 * (t // 128) reads the state of all keys < j0 = t0 - W_r and forms keys j0 .. t - W directly.
"""
import numpy as np

from oracle import rattn_oracle as orc


def bf16_round(x):
    """Round float64 values to the nearest bf16 (ties to even), returned as float64."""
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def _rms_bwd(x_saved, r, gam, dy):
    gy = gam[None, :] * dy
    return r[:, None] * gy - x_saved * (r[:, None] ** 3) * np.mean(gy * x_saved, axis=1, keepdims=True)


ROUNDING_POINTS = ("p", "phi", "c", "states", "saved", "out", "dx", "ds", "dc", "rstates", "grads")


def model_fwd_bwd(q, k, v, dO, W, scale=1.0, eps=1e-6, gamma_swa=None, gamma_rla=None, with_bwd=True,
                  exact=(), feature_map="softmax"):
    """Forward and backward of the layer with the matrix-core path's roundings.  q [B,T,Hq,D], k/v [B,T,Hkv,D]
    float64 holding bf16-representable values; feature_map "softmax" or "relu".
    `exact`: names from ROUNDING_POINTS whose rounding is switched off (to attribute the error to its sources).
    Returns dict(o, xs, xr, dq, dk, dv) (float64 arrays holding bf16-representable values)."""
    def rnd(name):
        return (lambda x: np.asarray(x, np.float64)) if name in exact else bf16_round
    r_p, r_phi, r_c, r_st, r_sv, r_out = rnd("p"), rnd("phi"), rnd("c"), rnd("states"), rnd("saved"), rnd("out")
    r_dx, r_ds, r_dc, r_rst, r_g = rnd("dx"), rnd("ds"), rnd("dc"), rnd("rstates"), rnd("grads")
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    if q.shape[1] % 128 != 0:
        # the kernels run ragged lengths on zero-padded copies (the layer is causal, zero rows of dO add nothing)
        T0 = q.shape[1]
        pad = lambda a: None if a is None else np.concatenate(
            [np.asarray(a, np.float64), np.zeros((a.shape[0], -T0 % 128) + a.shape[2:])], axis=1)
        out = model_fwd_bwd(pad(q), pad(k), pad(v), pad(dO), W, scale, eps, gamma_swa, gamma_rla, with_bwd, exact,
                            feature_map)
        return {n: a[:, :T0] for n, a in out.items()}
    B, T, Hq, D = q.shape
    Hkv = k.shape[2]; G = Hq // Hkv
    gs = orc._gains(gamma_swa, Hq, D); gr = orc._gains(gamma_rla, Hq, D)
    Wt = min(W, T)
    Wr = (Wt + 63) // 64 * 64
    t = np.arange(T)[:, None]; s = np.arange(T)[None, :]
    win = (s <= t) & (s > t - W)
    res = s <= t - W
    j0 = (t // 128) * 128 - Wr                      # first key the query's tile forms directly
    via_state = res & (s < j0)
    direct = res & ~via_state
    # backward, key side: key tile s0 = 128 * (s // 128) takes queries t >= s0 + 128 + Wr from the reverse state
    via_rstate = res & (t >= (s // 128) * 128 + 128 + Wr)
    direct_k = res & ~via_rstate
    out = {n: np.zeros_like(q) for n in ("o", "xs", "xr", "dq")}
    out["dk"] = np.zeros_like(k); out["dv"] = np.zeros_like(v)
    for b in range(B):
        for g in range(Hkv):
            kk = k[b, :, g]; vv = v[b, :, g]
            kf32 = orc.phi(kk, feature_map)
            kf = r_phi(kf32)
            # chunk states: fp32 prefix sums of bf16 products, rounded once when stored
            cs = np.cumsum(kf[:, :, None] * vv[:, None, :], axis=0)       # cs[n] = sum_{s <= n}
            dk_g = np.zeros((T, D)); dv_g = np.zeros((T, D)); dkf_g = np.zeros((T, D))
            per_head = []
            for hh in range(G):
                h = g * G + hh
                qq = q[b, :, h]
                qf32 = orc.phi(qq, feature_map)
                qf = r_phi(qf32)
                a = np.where(win, scale * (qq @ kk.T), -np.inf)
                m = a.max(axis=1, keepdims=True)
                e = np.exp(a - m)
                z = e.sum(axis=1, keepdims=True)
                p = e / z
                lse = (m + np.log(z))[:, 0]
                x_s = r_p(p) @ vv
                c = np.where(direct, r_c(qf @ kf.T), 0.0)
                x_r = c @ vv
                for t0 in range(0, T, 128):
                    jj = t0 - Wr
                    if jj > 0:
                        x_r[t0:t0 + 128] += qf[t0:t0 + 128] @ r_st(cs[jj - 1])
                r_s = 1.0 / np.sqrt(np.mean(x_s * x_s, axis=1) + eps)
                r_r = 1.0 / np.sqrt(np.mean(x_r * x_r, axis=1) + eps)
                out["o"][b, :, h] = r_out(gs[h] * x_s * r_s[:, None] + gr[h] * x_r * r_r[:, None])
                xs_sv = r_sv(x_s); xr_sv = r_sv(x_r)
                out["xs"][b, :, h] = xs_sv; out["xr"][b, :, h] = xr_sv
                if not with_bwd:
                    continue
                dy = np.asarray(dO, np.float64)[b, :, h]
                dxs = r_dx(_rms_bwd(xs_sv, r_s, gs[h], dy))
                dxr = r_dx(_rms_bwd(xr_sv, r_r, gr[h], dy))
                delta = np.sum(dxs * xs_sv, axis=1, keepdims=True)
                p_b = r_p(p)
                dp = dxs @ vv.T
                ds = r_ds(np.where(win, p * (dp - delta) * scale, 0.0))
                dq_h = ds @ kk
                dk_g += ds.T @ qq
                dv_g += p_b.T @ dxs
                # linear branch, query side: directly formed pairs + state
                dc = r_dc(np.where(direct, dxr @ vv.T, 0.0))
                dqf = dc @ kf
                for t0 in range(0, T, 128):
                    jj = t0 - Wr
                    if jj > 0:
                        dqf[t0:t0 + 128] += dxr[t0:t0 + 128] @ r_st(cs[jj - 1]).T
                dq_h += orc.phi_bwd(qq, qf32, dqf, feature_map)
                out["dq"][b, :, h] = r_g(dq_h)
                # key side: directly formed pairs now, the rest through the reverse states below
                ck = np.where(direct_k, r_c(qf @ kf.T), 0.0)
                dck = r_dc(np.where(direct_k, dxr @ vv.T, 0.0))
                dv_g += ck.T @ dxr
                dkf_g += dck.T @ qf
                per_head.append((qf, dxr))
            if with_bwd:
                # reverse states: R[s0] = sum_{t >= s0 + 128 + Wr} sum_heads phi(q_t)^T dx^r_t, [feature, value]
                for s0 in range(0, T, 128):
                    t_lo = s0 + 128 + Wr
                    if t_lo >= T:
                        continue
                    R = np.zeros((D, D))
                    for qf, dxr in per_head:
                        R += qf[t_lo:].T @ dxr[t_lo:]
                    R = r_rst(R)
                    sl = slice(s0, s0 + 128)
                    valid = (np.arange(s0, s0 + 128) <= T - 1 - W)[:, None]   # keys that any query reads
                    dv_g[sl] += np.where(valid, kf[sl] @ R, 0.0)
                    dkf_g[sl] += np.where(valid, vv[sl] @ R.T, 0.0)
                dk_g += orc.phi_bwd(kk, kf32, dkf_g, feature_map)
                out["dk"][b, :, g] = r_g(dk_g)
                out["dv"][b, :, g] = r_g(dv_g)
    return out
