"""CPU oracle for the deferred logit-lens projection and the steering pair.

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, fp64 NumPy statement
of what the method computes.  It is imported by the tests, by the smoke check
and by the benchmark's CPU-baseline leg, and by nothing else; it shares no
code, constant or helper with the HIP library and never calls it.

What it follows
  * Logit-lens projection, paper Sec. 3.3 Eq. (1): z = W_out . LN(h) + b, with
    LN the model's final normalisation layer (read here as RMSNorm with weight
    gamma and eps inside the square root) and b = 0.
  * Top-k extraction, paper Sec. 3.3 "Top-k extraction": the k largest logits
    per token by an argsort.  Ties: descending logit, ascending id.
  * Probabilities: full-vocabulary softmax (the paper's own variant, a softmax
    over the k selected logits only, is `topk_renormalised` below: an exact
    function of the full-softmax result).
  * Target log-probability and softmax entropy: the textbook definitions.
  * Steering direction, paper Sec. 3.4 Eq. (2): v = (y+ - y-)/||y+ - y-||_2,
    with y+/y- read as the means of the target/base rows.
  * Steering injection, paper Sec. 3.4 Eq. (3): h' = h + alpha v, applied
    after the normalisation: h' = RMSNorm(h) + alpha v.

Precision reading: the hidden states, gamma and W_out are bf16 bit patterns
(uint16).  They are widened exactly to fp64.  The normalised row is rounded
ONCE, round-to-nearest-even, from fp64 straight to bf16 before the product
with W_out (the contraction's inputs are bf16); `round_a=False` skips that
rounding and gives the un-rounded reference that is reported, not gated.
Everything after the rounding is fp64.

Pins (tests/test_oracle_pins.py): pure-Python brute force on tiny inputs, the
one-hot closed form, the zero-row uniform case, scale invariance, library
routines (scipy logsumexp / entropy, torch.topk, torch's bf16 cast), softmax
invariants, linearity of the logits in alpha, and planted-mistake variants
that each fail at least one pin.  The paper prints no numeric projection
result, so beyond those pins parity is unpinned by the paper itself.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits_to_f64",
    "f64_to_bf16_bits",
    "rmsnorm",
    "full_logits",
    "softmax_summaries",
    "lens_project",
    "topk_renormalised",
    "steer_vector",
    "steer_inject",
    "steer_sweep",
    "steer_inject_raw",
    "concat_trajectories",
]


# --------------------------------------------------------------------------
# bf16 <-> fp64.  bf16 = sign(1) exponent(8) fraction(7): the top half of an
# IEEE binary32 word.
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x) -> np.ndarray:
    """Round fp64 to bf16 (round-to-nearest, ties-to-even) in ONE step.

    Not via fp32: rounding twice can land on a different bf16 value.  A bf16
    number has 8 significant bits, so with x = m * 2**e, 0.5 <= |m| < 1, the
    spacing of bf16 numbers around x is 2**(e-8) (2**-133 in the subnormal
    range).  x / spacing is exact (a power-of-two scaling), np.rint rounds
    half to even, and the product back is exact as well.
    """
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    e = np.maximum(e, -125)                      # below 2**-126: fixed spacing
    spacing = np.ldexp(1.0, e - 8)
    q = np.rint(x / spacing) * spacing
    bf16_max = (2.0 - 2.0 ** -7) * 2.0 ** 127
    q = np.where(np.abs(q) > bf16_max, np.copysign(np.inf, q), q)
    q = np.where(np.isfinite(x), q, x)           # inf / nan pass through
    # q is exactly representable in binary32 now; keep its top 16 bits.
    return (q.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# Projection (Eq. 1) and its summaries
# --------------------------------------------------------------------------
def rmsnorm(hidden_bits, gamma_bits, eps: float, round_a: bool = True) -> np.ndarray:
    """Final normalisation of Eq. (1): a_j = gamma_j * h_j / sqrt(mean_j h_j^2 + eps).

    hidden_bits [R, d] uint16, gamma_bits [d] uint16 or None.  gamma None means
    the rows are already normalised (the output of `steer_inject`) and are
    passed through unchanged.  Returns fp64 [R, d]; with round_a the values are
    those of the bf16 numbers nearest to the fp64 result.
    """
    h = bf16_bits_to_f64(hidden_bits)
    if gamma_bits is None:
        return h
    g = bf16_bits_to_f64(gamma_bits)
    ms = np.mean(h * h, axis=-1, keepdims=True)
    a = g * h / np.sqrt(ms + float(eps))
    if round_a:
        a = bf16_bits_to_f64(f64_to_bf16_bits(a))
    return a


def full_logits(a: np.ndarray, w_bits, slab: int = 8192, bias=None) -> np.ndarray:
    """z[r, v] = sum_j a[r, j] * W_out[v, j] + b[v]  (Eq. 1; b = 0 when bias is None), fp64 [R, V].

    W_out is widened to fp64 one slab of vocabulary rows at a time so that a
    2 GB bf16 matrix never becomes a 17 GB fp64 one; the slabs are disjoint
    column blocks of z, so this is the plain product, not a reordering of it.
    """
    w_bits = np.asarray(w_bits)
    V = w_bits.shape[0]
    z = np.empty((a.shape[0], V), dtype=np.float64)
    for v0 in range(0, V, slab):
        w = bf16_bits_to_f64(w_bits[v0:v0 + slab])
        z[:, v0:v0 + slab] = a @ w.T
    if bias is not None:
        z += np.asarray(bias, dtype=np.float64)[None, :]
    return z


def softmax_summaries(z: np.ndarray, k: int, target_ids=None) -> dict:
    """Exact softmax summaries of full logits z [R, V] (fp64).

    lse = log sum_v exp z_v (shifted by the row maximum), p_v = exp(z_v - lse),
    entropy = -sum_v p_v log p_v, target_logp = z_target - lse, and the k
    largest logits by a stable sort on (-z, id): descending logit, ascending id
    among equals.  Also returns the (k+1) largest logits, which the parity
    tests use to find near-ties.
    """
    R, V = z.shape
    if not 1 <= k <= V:
        raise ValueError("need 1 <= k <= V")
    zmax = np.max(z, axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.sum(np.exp(z - zmax), axis=1))
    logp = z - lse[:, None]
    p = np.exp(logp)
    # 0 * (-inf) cannot occur for finite logits; p underflowing to 0 adds 0.
    entropy = -np.sum(np.where(p > 0.0, p * logp, 0.0), axis=1)
    order = np.argsort(-z, axis=1, kind="stable")       # ties keep ascending id
    kk = min(k + 1, V)
    top = order[:, :kk]
    top_z = np.take_along_axis(z, top, axis=1)
    out = {
        "topk_ids": top[:, :k].astype(np.int32),
        "topk_p": np.take_along_axis(p, top[:, :k], axis=1),
        "topk_logits": top_z[:, :k],
        "top_logits_k1": top_z,                           # k+1 (or V) largest
        "lse": lse,
        "entropy": entropy,
    }
    if target_ids is not None:
        t = np.asarray(target_ids, dtype=np.int64)
        ok = (t >= 0) & (t < V)
        zt = z[np.arange(R), np.where(ok, t, 0)]
        out["target_logp"] = np.where(ok, zt - lse, np.nan)
    return out


def lens_project(hidden_bits, gamma_bits, w_bits, eps: float, k: int,
                 target_ids=None, round_a: bool = True, bias=None) -> dict:
    """The whole projection for rows hidden_bits [R, d]: Eq. (1), then the summaries."""
    a = rmsnorm(hidden_bits, gamma_bits, eps, round_a=round_a)
    z = full_logits(a, w_bits, bias=bias)
    return softmax_summaries(z, k, target_ids)


def topk_renormalised(topk_p: np.ndarray) -> np.ndarray:
    """The paper's own probabilities (Sec. 3.3): softmax over the k selected logits only.

    exp(z_i) / sum_{j in top-k} exp(z_j) = p_i / sum_{j in top-k} p_j.
    """
    topk_p = np.asarray(topk_p, dtype=np.float64)
    return topk_p / np.sum(topk_p, axis=-1, keepdims=True)


# --------------------------------------------------------------------------
# Steering (Eq. 2, Eq. 3)
# --------------------------------------------------------------------------
def steer_vector(base_bits, target_bits, normalize: bool = True) -> np.ndarray:
    """Eq. (2) with y+ / y- the column means of the target / base rows; fp64 [d].

    A zero difference has no direction: the zero vector is returned.
    """
    yb = np.mean(bf16_bits_to_f64(base_bits), axis=0)
    yt = np.mean(bf16_bits_to_f64(target_bits), axis=0)
    diff = yt - yb
    if not normalize:
        return diff
    nrm = np.sqrt(np.sum(diff * diff))
    if nrm == 0.0:
        return np.zeros_like(diff)
    return diff / nrm


def steer_inject(hidden_bits, gamma_bits, eps: float, v, alpha: float) -> np.ndarray:
    """Eq. (3) after the normalisation: bf16( RMSNorm(h) + alpha * v ), as uint16 bits.

    The norm is NOT rounded on its own here: the only rounding is the final one
    to the bf16 output.  `v` is taken as given (fp32 or fp64 values).
    """
    a = rmsnorm(hidden_bits, gamma_bits, eps, round_a=False)
    out = a + float(alpha) * np.asarray(v, dtype=np.float64)[None, :]
    return f64_to_bf16_bits(out)


def steer_sweep(hidden_bits, gamma_bits, w_bits, eps: float, v, alphas, target_ids=None, round_a: bool = True,
                k: int = 1) -> dict:
    """Lens read-out of Eq. (3) for several steering strengths (Sec. 3.4, dose-response of Sec. 5).

    For every alpha: z_alpha = W_U (a + alpha v) with a the normalised row (rounded to bf16
    once, as in lens_project, when round_a), written out as the definition says: the steered
    rows are formed first, in fp64 and without any further rounding, then multiplied by W_U.
    Returns, per alpha and row, the arg max (smallest id on ties), its full-softmax
    probability, the target log-probability and the entropy: arrays of shape [n_alpha, R];
    and the k most likely tokens with their probabilities and logits (the paper's figures
    list k = 3 per cell), sorted as in softmax_summaries: arrays of shape [n_alpha, R, k].
    """
    a = rmsnorm(hidden_bits, gamma_bits, eps, round_a=round_a) if gamma_bits is not None else bf16_bits_to_f64(hidden_bits)
    vv = np.asarray(v, dtype=np.float64)
    out = {"top1_ids": [], "top1_p": [], "target_logp": [], "entropy": [], "topk_ids": [], "topk_p": [], "topk_logits": []}
    for alpha in alphas:
        z = full_logits(a + float(alpha) * vv[None, :], w_bits)
        sm = softmax_summaries(z, k, target_ids)
        out["top1_ids"].append(sm["topk_ids"][:, 0])
        out["top1_p"].append(sm["topk_p"][:, 0])
        out["topk_ids"].append(sm["topk_ids"])
        out["topk_p"].append(sm["topk_p"])
        out["topk_logits"].append(sm["topk_logits"])
        if target_ids is not None:
            out["target_logp"].append(sm["target_logp"])
        out["entropy"].append(sm["entropy"])
    return {name: np.stack(x) for name, x in out.items() if x}


def steer_inject_raw(hidden_bits, v, alpha: float, layer_scale: float = 1.0, clip_ratio: float = 0.0) -> np.ndarray:
    """h' = h + alpha v inside the model (Sec. 3.4, the equation after Eq. 2), with the two
    safeguards its stability paragraph names but does not define.  Reading taken here:
    s = alpha * layer_scale is the strength at this layer, and its magnitude is clipped to
    clip_ratio * ||h_r||_2 row by row (clip_ratio <= 0: no clipping); the shifted row is
    rounded to bf16 once.  Returns uint16 bits.  Parity unpinned by the paper (it prints no
    formula); pinned against the plain equation and the clipping bound.
    """
    h = bf16_bits_to_f64(hidden_bits)
    s = float(alpha) * float(layer_scale)
    if clip_ratio > 0:
        cap = float(clip_ratio) * np.sqrt(np.sum(h * h, axis=-1, keepdims=True))
        beta = np.sign(s) * np.minimum(abs(s), cap)
    else:
        beta = np.full(h.shape[:-1] + (1,), s)
    return f64_to_bf16_bits(h + beta * np.asarray(v, dtype=np.float64)[None, :])


def concat_trajectories(step_slices, L: int, C: int) -> np.ndarray:
    """Stage 3's first step (Sec. 3.1; Alg. 1, Phase 2): the slices recorded during generation,
    each of shape [L*C, n_i, d] for the n_i newest tokens ((layer, type)-major), concatenated
    along the token axis into the trajectories H[l, c, :, :] of shape [L, C, T, d].
    """
    full = np.concatenate([np.asarray(x) for x in step_slices], axis=1)     # [L*C, T, d]
    return full.reshape(L, C, full.shape[1], full.shape[2])

