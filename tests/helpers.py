"""Shared test helpers (no method arithmetic: conversions and the error metric)."""
import numpy as np
import torch

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 8e-3}   # max over images of relative L2 error vs the fp64 oracle
TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def f64(t):
    """torch tensor (any float dtype, any device) -> numpy float64, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def bits_as_f64(t):
    """Element bit patterns as float64 integers (exact), for bit-exactness checks
    of pure data movement through the value-agnostic oracle routines."""
    t = t.detach().to("cpu").contiguous()
    it = torch.int16 if t.element_size() == 2 else torch.int32
    return t.view(it).to(torch.float64).numpy()


def bits(t):
    t = t.detach().to("cpu").contiguous()
    it = torch.int16 if t.element_size() == 2 else torch.int32
    return t.view(it).numpy()


def rel_l2_per_image(y, ref):
    """max over images n of ||y[n]-ref[n]||_2 / ||ref[n]||_2 (float64 numpy inputs)."""
    y = y.reshape(y.shape[0], -1)
    ref = ref.reshape(ref.shape[0], -1)
    num = np.sqrt(((y - ref) ** 2).sum(axis=1))
    den = np.sqrt((ref ** 2).sum(axis=1))
    den = np.where(den == 0, 1.0, den)
    return float((num / den).max())


# --- element-wise bound ------------------------------------------------------------------------
# A result computed with exact products, fp32 accumulation in any order and one rounding to the
# output type differs from the exact value v by at most
#     acc + ulp_out(|v| + acc) / 2,     acc = 2 (K + 2) 2^-24 S,
# where S = sum |x| |w| + |b| over the element's taps (the oracle run on absolute values) and K the
# number of taps: every addition (and, for fp32 operands, every product) contributes at most one
# fp32 rounding of a partial sum that S bounds.  A dropped, doubled or misplaced tap changes the
# element by about S / K, orders of magnitude above this.
_MANT = {"f32": 23, "f16": 10, "bf16": 7}
_EMIN = {"f32": -126, "f16": -14, "bf16": -126}


def ulp_out(v, dt):
    """Spacing of the output type's grid at magnitude |v| (float64 numpy array)."""
    _, ex = np.frexp(np.abs(v))                      # |v| = m * 2^ex, m in [0.5, 1)
    e = np.maximum(ex - 1, _EMIN[dt])
    return np.ldexp(1.0, e - _MANT[dt])


def elementwise_bound(ref, S, K, dt):
    acc = 2.0 * (K + 2) * 2.0 ** -24 * S
    return acc + 0.5 * ulp_out(np.abs(ref) + acc, dt)


def assert_elementwise(y, ref, S, K, dt, what=""):
    """Every element of y within the bound above of ref; names the worst element on failure."""
    bound = elementwise_bound(ref, S, K, dt)
    excess = np.abs(y - ref) / bound
    worst = np.unravel_index(int(np.argmax(excess)), excess.shape)
    assert excess[worst] <= 1.0, "%s: element %s: got %.9g, oracle %.9g, |diff| %.3e > bound %.3e (%d elements beyond)" % (
        what, tuple(int(i) for i in worst), y[worst], ref[worst], abs(y[worst] - ref[worst]), bound[worst],
        int((excess > 1.0).sum()))
    return float(excess[worst])


def assert_same_to_rounding(a, b, S, K, dt, what="", max_fraction=0.05):
    """Two walks of the same sum (other fp32 order): no element further apart than one output
    spacing plus twice the accumulation bound; for 16-bit outputs only a few elements differ at all."""
    acc = 2.0 * (K + 2) * 2.0 ** -24 * S
    bound = ulp_out(np.maximum(np.abs(a), np.abs(b)), dt) + 2.0 * acc
    d = np.abs(a - b)
    excess = d / bound
    worst = np.unravel_index(int(np.argmax(excess)), excess.shape)
    assert excess[worst] <= 1.0, "%s: element %s: %.9g vs %.9g, |diff| %.3e > %.3e" % (
        what, tuple(int(i) for i in worst), a[worst], b[worst], d[worst], bound[worst])
    if dt != "f32":
        frac = float((d != 0).mean())
        assert frac <= max_fraction, "%s: %.2f %% of the elements differ" % (what, 100 * frac)
