"""Tolerances of the parity contract, written once for the CPU and GPU tests.

Integer work, the fold and the pack of a given fp32 value are bit-exact.  The
fp32 master parameter and the two moments must agree with the fp64 reference
within 1e-6 relative.  Where a result is the difference of two terms that may
cancel (the first moment changing sign, a parameter of the size of the step),
"relative" is taken against the magnitude of the terms, not of the difference.
"""
import numpy as np

REL = 1e-6


def check_moments_and_params(got_p, got_m, got_v, ref_p, ref_m, ref_v, *, p_old, m_old, g_hat,
                             beta1=0.9, beta2=0.999, what="", hist=None, g_terms=None, v_old=None, l2=None):
    """All arrays fp32 (got_*: path under test; ref_*: fp64 evaluation rounded once);
    g_hat = scaled, clipped gradient as fp64.  In a run of several steps each side
    carries its own state, so a rounding made when the terms were large is still
    there after they have cancelled: pass the same dict as `hist` at every step and
    the term magnitudes become running maxima over the run.
    g_terms: with classic L2 decay the gradient that enters the moments is itself a sum that
    may cancel, scale * g + wd * p; pass |scale * g| + |wd * p| (fp64) and the second moment,
    quadratic in that sum, is judged against the terms too (v_old: its old value, default 0).
    l2 = dict(step_size, sqrt_bc2, eps): then the parameter's tolerance also carries what an
    error of 1e-6 * g_terms in that sum does to the step, by first-order propagation through
    q = m / (sqrt(v) / sqrt_bc2 + eps)."""
    b1 = float(np.float32(beta1))
    ref_p64, ref_m64, ref_v64 = (a.astype(np.float64) for a in (ref_p, ref_m, ref_v))
    mag_g = np.abs(g_hat) if g_terms is None else np.maximum(np.abs(g_hat), g_terms)
    floor_m = np.abs(b1 * m_old.astype(np.float64)) + (1 - b1) * mag_g
    floor_v = np.abs(ref_v64)
    if g_terms is not None:
        b2 = float(np.float32(beta2))
        old = 0.0 if v_old is None else np.abs(b2 * v_old.astype(np.float64))
        floor_v = np.maximum(floor_v, old + (1 - b2) * mag_g * mag_g)
    tol_v = REL * floor_v
    floor_p = np.abs(p_old.astype(np.float64)) + np.abs(ref_p64 - p_old.astype(np.float64))
    floor_p = np.maximum(np.abs(ref_p64), floor_p)
    floor_m = np.maximum(np.abs(ref_m64), floor_m)
    if hist is not None:
        floor_p = hist["p"] = np.maximum(hist.get("p", 0.0), floor_p)
        floor_m = hist["m"] = np.maximum(hist.get("m", 0.0), floor_m)
    tol_p = REL * floor_p
    tol_m = REL * floor_m
    if g_terms is not None and l2 is not None:
        b2 = float(np.float32(beta2))
        d_g = REL * mag_g
        root_v = np.sqrt(np.maximum(ref_v64, 0.0))
        den = root_v / l2["sqrt_bc2"] + l2["eps"]
        q = np.abs(ref_m64) / den
        d_q = d_g * ((1 - b1) / den + q * (1 - b2) * np.abs(g_hat) / (den * l2["sqrt_bc2"] * np.maximum(root_v, 1e-300)))
        tol_p = tol_p + l2["step_size"] * d_q
    for name, got, ref, tol in (("m", got_m, ref_m64, tol_m), ("v", got_v, ref_v64, tol_v),
                                ("p", got_p, ref_p64, tol_p)):
        bad = np.abs(got.astype(np.float64) - ref) > tol
        if bad.any():
            k = int(np.argmax(bad))
            raise AssertionError(f"{what} {name}[{k}]: got {got[k]!r} want {ref[k]!r} tol {tol[k]:.3e} "
                                 f"({int(bad.sum())} of {bad.size} outside 1e-6)")
    return tol_p


def ulp_distance_f32(a, b):
    """Largest distance in units in the last place between two fp32 arrays."""
    ia = a.view(np.int32).astype(np.int64)
    ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7FFFFFFF), ia)
    ib = np.where(ib < 0, -(ib & 0x7FFFFFFF), ib)
    return int(np.max(np.abs(ia - ib))) if a.size else 0


def check_bf16_within_one_ulp(got_bits, ref_bits, what="", ref_p=None, tol_p=None, fmt="bf16"):
    """bf16 bit patterns (uint16) at most one unit in the last place apart.  Where the
    parameter itself is a cancelled difference (its 1e-6 tolerance tol_p, taken on the
    terms, is large against its own size) one bf16 ulp of the tiny result means nothing:
    there the packed value must lie within tol_p plus one bf16 rounding of the reference."""
    def key(h):
        i = h.astype(np.int32)
        return np.where(i & 0x8000, -(i & 0x7FFF), i)
    d = np.abs(key(got_bits) - key(ref_bits))
    bad = d > 1
    if bad.any() and ref_p is not None:
        if fmt == "f16":
            val = np.ascontiguousarray(got_bits).view(np.float16).astype(np.float64)
            eps = 2.0 ** -11
        else:
            val = (got_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            eps = 2.0 ** -8
        ref = ref_p.astype(np.float64)
        ok = np.abs(val - ref) <= tol_p + eps * np.maximum(np.abs(ref), np.abs(val)) + (2.0 ** -25 if fmt == "f16" else 0)
        bad &= ~ok
    assert not bad.any(), f"{what} packed bf16 differs by {int(d[bad].max())} ulp"
