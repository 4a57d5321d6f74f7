"""Pure-Python (no NumPy) statement of the projection, for tiny inputs only.

Used to pin the NumPy oracle: triple loops, math.fsum, math.exp, sorted().
Inputs are Python floats (already widened from bf16 by the caller) so this
file has no bit tricks at all; the bf16 rounding of the normalised row is
done with the struct module.
"""
import math
import struct


def round_to_bf16(x: float) -> float:
    """Nearest bf16 value to a Python float (ties to even), via exact integer arithmetic."""
    if x == 0.0 or math.isinf(x) or math.isnan(x):
        return x
    m, e = math.frexp(abs(x))            # abs(x) = m * 2**e, 0.5 <= m < 1
    e = max(e, -125)
    # abs(x) / 2**(e-8) as an exact fraction, then round half to even.
    scaled = abs(x) / math.ldexp(1.0, e - 8)     # exact: power-of-two scaling
    lo = math.floor(scaled)
    frac = scaled - lo
    if frac > 0.5 or (frac == 0.5 and lo % 2 == 1):
        lo += 1
    r = math.ldexp(float(lo), e - 8)
    # sanity: representable in binary32 with 16 low zero bits
    bits = struct.unpack("<I", struct.pack("<f", r))[0]
    assert bits & 0xFFFF == 0
    return math.copysign(r, x)


def project_row(h, gamma, W, eps, k, target, round_a=True, bias=None):
    """One lens row.  h [d], gamma [d] or None, W [V][d] (lists of floats).

    Returns dict(ids, p, logits, lse, entropy, target_logp).
    """
    d = len(h)
    V = len(W)
    if gamma is None:
        a = list(h)
    else:
        ms = math.fsum(x * x for x in h) / d
        a = [gamma[j] * h[j] / math.sqrt(ms + eps) for j in range(d)]
        if round_a:
            a = [round_to_bf16(x) for x in a]
    z = [math.fsum([a[j] * W[v][j] for j in range(d)] + ([bias[v]] if bias is not None else [])) for v in range(V)]
    zmax = max(z)
    lse = zmax + math.log(math.fsum(math.exp(x - zmax) for x in z))
    p = [math.exp(x - lse) for x in z]
    entropy = -math.fsum(pi * (zi - lse) for pi, zi in zip(p, z) if pi > 0.0)
    order = sorted(range(V), key=lambda v: (-z[v], v))[:k]
    return {
        "ids": order,
        "p": [p[v] for v in order],
        "logits": [z[v] for v in order],
        "lse": lse,
        "entropy": entropy,
        "target_logp": (z[target] - lse) if 0 <= target < V else float("nan"),
    }


def steer_vector(base, target, normalize=True):
    """Difference of the row means of target and base, L2-normalised."""
    d = len(base[0])
    yb = [math.fsum(r[j] for r in base) / len(base) for j in range(d)]
    yt = [math.fsum(r[j] for r in target) / len(target) for j in range(d)]
    diff = [yt[j] - yb[j] for j in range(d)]
    if not normalize:
        return diff
    n = math.sqrt(math.fsum(x * x for x in diff))
    return [0.0] * d if n == 0.0 else [x / n for x in diff]
