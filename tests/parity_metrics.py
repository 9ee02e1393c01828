"""Error metrics and bounds shared by the GPU parity tests (test infrastructure; no arithmetic of the method).

Outputs (bf16, unit scale after the two RMS norms): the bar is max-abs 2e-2.  A bf16 number of magnitude 4..8 cannot
be stored closer than 2^-6 = 0.0156 to an arbitrary real, so two figures are asserted:
  * the raw max-abs error over all elements with |ref| < 4 (no allowance at all), and
  * over all elements, the error beyond the stored value's own rounding, |err| - half_ulp_bf16(ref).
The raw maximum over everything is returned too and printed by the tests.

Gradients (bf16) on the matrix-core path: every contraction takes bf16 operands.  tests/bf16_error_model.py repeats the
oracle's arithmetic with exactly those roundings; tests/test_error_model.py shows on the CPU that this alone gives
RMS(err)/RMS(ref) = 2.6e-3 .. 3.5e-3 and a worst element (beyond its own storage rounding) of up to 4.3e-2 of RMS(ref)
on seeded random shapes, i.e. that the 2e-2-of-RMS figure cannot be met by any implementation that feeds bf16 operands to
the matrix cores and stores bf16 gradients.  The GPU tests therefore assert
  * against the model evaluated on the SAME input (no seed choice involved): RMS error <= 1.2 x the model's; the
    share of elements whose error exceeds 1e-2 of RMS(ref) <= 3 x the model's share (+ 5e-4); worst element <= 3 x the
    model's worst element.  (The worst element is a maximum over 1e5..1e7 samples of rounding noise on the few rows
    that amplify it - rows just past the window, rows with few keys.  The kernels round un-normalised probabilities
    and the model normalised ones, i.e. on different grids, so the two draw different samples of that noise:
    over some 400 tensors compared the ratio of the two maxima ranged from 0.6 to 2.8, the RMS ratio from 0.94 to
    1.07.)  And
  * absolute caps, also where the model is too slow to evaluate (full-size tensors): GRAD_RMS_TOL and
    GRAD_WORST_TOL below = what the CPU sweep of the model supports, with the same head-room.
The general (fp32-arithmetic) kernels keep the 2e-2-of-RMS bar.
"""
import math

import numpy as np

OUT_TOL_BF16 = 2e-2      # max-abs, unit-scale outputs
GRAD_TOL_GENERAL = 2e-2  # worst element / RMS(ref), general kernels (fp32 arithmetic)
GRAD_RMS_TOL = 5e-3      # RMS(err) / RMS(ref), matrix-core path
GRAD_WORST_TOL = 8e-2    # worst (|err| - half_ulp_bf16(ref)) / RMS(ref), matrix-core path
MODEL_RMS_FACTOR = 1.2
MODEL_TAIL_FACTOR = 3.0   # on the share of elements with an error above TAIL_LEVEL * RMS(ref)
MODEL_WORST_FACTOR = 3.0
TAIL_LEVEL = 1e-2


def half_ulp_bf16(x):
    """Half the spacing of bf16 numbers at |x|: the largest error of storing the exact value x as bf16."""
    a = np.abs(np.asarray(x, np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return np.where(a > 0, 2.0 ** (e - 8), 0.0)


def out_err_bf16(got, ref):
    """dict(raw, raw_lt4, beyond_storage) for a bf16 output tensor `got` (float64 array) against the oracle."""
    e = np.abs(got - ref)
    small = np.abs(ref) < 4.0
    return dict(raw=float(e.max()), raw_lt4=float(e[small].max()) if small.any() else 0.0,
                beyond_storage=float(np.maximum(e - half_ulp_bf16(ref), 0.0).max()))


def assert_out_bf16(got, ref, gain_scale=1.0, what="o", tol=OUT_TOL_BF16):
    """Asserts the two output figures; `gain_scale` = max(1, max |gain|): the error of a gained output scales with
    the gain.  Returns the figures."""
    r = out_err_bf16(got, ref)
    print(f"{what}: raw max-abs {r['raw']:.4f}, raw where |ref|<4 {r['raw_lt4']:.4f}, beyond storage rounding "
          f"{r['beyond_storage']:.4f} (bound {tol * gain_scale:.4f})", flush=True)
    assert r["raw_lt4"] <= tol * gain_scale, f"{what}: raw max-abs error {r['raw_lt4']} where |ref| < 4"
    assert r["beyond_storage"] <= tol * gain_scale, f"{what}: error beyond storage rounding {r['beyond_storage']}"
    return r


def grad_err_bf16(got, ref):
    """dict(raw = max|err|/RMS(ref), worst = max(|err| - half_ulp(ref))/RMS(ref), rms = RMS(err)/RMS(ref),
    tail = share of elements with (|err| - half_ulp(ref)) > TAIL_LEVEL * RMS(ref))."""
    rms = math.sqrt(float(np.mean(ref ** 2))) + 1e-300
    e = np.abs(got - ref)
    beyond = np.maximum(e - half_ulp_bf16(ref), 0.0)
    return dict(raw=float(e.max() / rms), worst=float(beyond.max() / rms),
                rms=math.sqrt(float(np.mean(e ** 2))) / rms, tail=float(np.mean(beyond > TAIL_LEVEL * rms)))


def assert_grad_bf16(got, ref, what, model=None, worst_tol=GRAD_WORST_TOL, rms_tol=GRAD_RMS_TOL):
    """Matrix-core path gradient check.  `model`: the same tensor from tests/bf16_error_model.py on the same input
    (None where it is too slow to evaluate: then only the absolute caps apply)."""
    if np.all(ref == 0):
        assert float(np.abs(got).max()) <= 1e-6, f"{what} must be zero"
        return None
    g = grad_err_bf16(got, ref)
    line = f"{what}: raw {g['raw']:.4f} worst {g['worst']:.4f} rms {g['rms']:.5f} tail {g['tail']:.2e}"
    if model is not None:
        m = grad_err_bf16(model, ref)
        line += f" | model raw {m['raw']:.4f} worst {m['worst']:.4f} rms {m['rms']:.5f} tail {m['tail']:.2e}"
    print(line, flush=True)
    assert g["rms"] <= rms_tol and g["worst"] <= worst_tol, line
    if model is not None:
        assert g["rms"] <= MODEL_RMS_FACTOR * m["rms"] + 1e-4, line
        assert g["tail"] <= MODEL_TAIL_FACTOR * m["tail"] + 5e-4, line
        assert g["worst"] <= MODEL_WORST_FACTOR * m["worst"] + 2e-3, line
    return g
