"""Pins for the CPU oracle: each checks it against something other than itself.

Every pin is a function of the oracle module `O`, so the same pins can be run
against deliberately broken copies (the `MUTANTS` at the bottom): the real
oracle must pass them all, and every planted mistake must fail at least one.
"""
import contextlib
import math
import struct

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import oracle.lens_oracle as ORACLE
from tests import brute_force as BF

LOG = math.log


# ----------------------------------------------------------------------------
# helpers (test side only)
# ----------------------------------------------------------------------------
def to_bits(x):
    """fp32-representable array -> bf16 bits via torch's own cast (a library routine)."""
    t = torch.tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_float(bits):
    """bf16 bits -> Python floats with struct (independent of the oracle's widening)."""
    flat = [struct.unpack("<f", struct.pack("<I", int(b) << 16))[0]
            for b in np.asarray(bits).ravel()]
    return np.array(flat, dtype=np.float64).reshape(np.asarray(bits).shape)


def rand_case(seed, R, d, V, scale=1.0):
    rng = np.random.default_rng(seed)
    h = to_bits(scale * rng.standard_normal((R, d)))
    g = to_bits(1.0 + 0.1 * rng.standard_normal(d))
    W = to_bits(0.5 * rng.standard_normal((V, d)))
    t = rng.integers(0, V, size=R)
    return h, g, W, t


# ----------------------------------------------------------------------------
# the pins
# ----------------------------------------------------------------------------
def pin_bf16_widen(O):
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4049, 0x0001, 0x7F7F, 0x8000, 0x3DCD], dtype=np.uint16)
    assert np.array_equal(O.bf16_bits_to_f64(bits), bits_to_float(bits))


def pin_bf16_round(O):
    # ties go to even; direct rounding from fp64 (not through fp32)
    cases = {
        1.0: 0x3F80,
        1.0 + 2.0 ** -8: 0x3F80,                     # tie -> even (down)
        1.0 + 3 * 2.0 ** -8: 0x3F82,                 # tie -> even (up)
        1.0 + 2.0 ** -8 + 2.0 ** -30: 0x3F81,        # just above a tie; via fp32 it would fall to 0x3F80
        -(1.0 + 2.0 ** -8 + 2.0 ** -30): 0xBF81,
        0.0: 0x0000,
        3.140625: 0x4049,
        2.0 ** -133: 0x0001,                         # smallest subnormal
        2.0 ** -134: 0x0000,                         # tie with zero -> even
        3.0e38: 0x7F62,
        3.4e38: 0x7F80,                              # overflows to +inf
    }
    xs = np.array(list(cases.keys()))
    want = np.array(list(cases.values()), dtype=np.uint16)
    got = O.f64_to_bf16_bits(xs)
    assert np.array_equal(got, want), (got, want)
    # on fp32-representable inputs it is torch's cast
    rng = np.random.default_rng(1)
    x32 = (rng.standard_normal(20000) * np.exp(rng.uniform(-30, 30, 20000))).astype(np.float32)
    assert np.array_equal(O.f64_to_bf16_bits(x32.astype(np.float64)), to_bits(x32))
    # brute-force rounding agrees on fp64 inputs that are not fp32-representable
    x64 = rng.standard_normal(500) * np.exp(rng.uniform(-5, 5, 500))
    want = to_bits(np.array([BF.round_to_bf16(float(v)) for v in x64]))
    assert np.array_equal(O.f64_to_bf16_bits(x64), want)


def pin_brute_force(O):
    for seed, (R, d, V, k) in enumerate([(3, 8, 11, 4), (2, 8, 8, 8), (4, 16, 5, 1)]):
        h, g, W, t = rand_case(seed, R, d, V)
        for round_a in (True, False):
            got = O.lens_project(h, g, W, 1e-5, k, t, round_a=round_a)
            hf, gf, Wf = bits_to_float(h), bits_to_float(g), bits_to_float(W)
            for r in range(R):
                want = BF.project_row(list(hf[r]), list(gf), [list(w) for w in Wf], 1e-5, k,
                                      int(t[r]), round_a=round_a)
                assert list(got["topk_ids"][r]) == want["ids"]
                np.testing.assert_allclose(got["topk_p"][r], want["p"], rtol=1e-12, atol=1e-15)
                np.testing.assert_allclose(got["topk_logits"][r], want["logits"], rtol=1e-12, atol=1e-13)
                assert abs(got["lse"][r] - want["lse"]) < 1e-12
                assert abs(got["entropy"][r] - want["entropy"]) < 1e-12
                assert abs(got["target_logp"][r] - want["target_logp"]) < 1e-12
        # gamma None = rows used as they are
        got = O.lens_project(h, None, W, 1e-5, k, t)
        want = BF.project_row(list(hf[0]), None, [list(w) for w in Wf], 1e-5, k, int(t[0]))
        assert list(got["topk_ids"][0]) == want["ids"]
        np.testing.assert_allclose(got["topk_p"][0], want["p"], rtol=1e-12)


def pin_bias(O):
    """Eq. (1) with its b: brute force, and a shift of every logit by a constant changes nothing but the logits."""
    h, g, W, t = rand_case(41, 3, 8, 13)
    rng = np.random.default_rng(2)
    b = rng.standard_normal(13)
    got = O.lens_project(h, g, W, 1e-5, 4, t, bias=b)
    hf, gf, Wf = bits_to_float(h), bits_to_float(g), bits_to_float(W)
    for r in range(3):
        want = BF.project_row(list(hf[r]), list(gf), [list(w) for w in Wf], 1e-5, 4, int(t[r]), bias=list(b))
        assert list(got["topk_ids"][r]) == want["ids"]
        np.testing.assert_allclose(got["topk_p"][r], want["p"], rtol=1e-12)
        assert abs(got["entropy"][r] - want["entropy"]) < 1e-12
        assert abs(got["target_logp"][r] - want["target_logp"]) < 1e-12
    base = O.lens_project(h, g, W, 1e-5, 4, t)
    shifted = O.lens_project(h, g, W, 1e-5, 4, t, bias=np.full(13, 2.5))
    assert np.array_equal(base["topk_ids"], shifted["topk_ids"])
    np.testing.assert_allclose(base["topk_p"], shifted["topk_p"], rtol=1e-12)
    np.testing.assert_allclose(shifted["topk_logits"], base["topk_logits"] + 2.5, rtol=1e-12)
    # a huge bias on one id puts it first
    b2 = np.zeros(13); b2[7] = 100.0
    assert np.all(O.lens_project(h, g, W, 1e-5, 4, t, bias=b2)["topk_ids"][:, 0] == 7)


def pin_invariants(O):
    h, g, W, t = rand_case(7, 12, 64, 300)
    k = 9
    out = O.lens_project(h, g, W, 1e-5, k, t)
    z = O.full_logits(O.rmsnorm(h, g, 1e-5), W)
    p_full = np.exp(z - out["lse"][:, None])
    assert np.all(np.abs(p_full.sum(1) - 1.0) < 1e-12)
    assert np.all(out["entropy"] >= 0) and np.all(out["entropy"] <= LOG(300) + 1e-12)
    assert np.all(np.diff(out["topk_p"], axis=1) <= 0)
    assert np.all(out["topk_p"].sum(1) <= 1 + 1e-12)
    assert np.all(out["target_logp"] <= 1e-15)
    # the k reported are the k largest of the row, and there are exactly V-k not larger
    for r in range(12):
        kth = out["topk_logits"][r, -1]
        assert np.sum(z[r] > kth) <= k - 1
        assert len(set(out["topk_ids"][r])) == k
        np.testing.assert_allclose(z[r, out["topk_ids"][r]], out["topk_logits"][r], rtol=0, atol=0)
    # target inside the top-k: its log-prob is the log of the listed probability
    t2 = out["topk_ids"][:, 2]
    out2 = O.lens_project(h, g, W, 1e-5, k, t2)
    np.testing.assert_allclose(out2["target_logp"], np.log(out2["topk_p"][:, 2]), atol=1e-12)
    # target outside [0, V): NaN, no exception
    out3 = O.lens_project(h, g, W, 1e-5, k, np.array([-1, 300] + [0] * 10))
    assert np.isnan(out3["target_logp"][0]) and np.isnan(out3["target_logp"][1])
    assert np.isfinite(out3["target_logp"][2])


def pin_one_hot(O):
    """h = c e_j, gamma = 1: the logits are a scaled column of W_out."""
    d, V, k, j = 256, 97, 6, 37
    rng = np.random.default_rng(3)
    Wf = (0.02 * rng.standard_normal((V, d))).astype(np.float32)
    W = to_bits(Wf)
    Wcol = bits_to_float(W)[:, j]
    for c, eps in [(4.0, 1e-30), (-0.5, 1e-30), (2.0, 1e-5)]:
        h = np.zeros((1, d), dtype=np.float32)
        h[0, j] = c
        s = math.copysign(1.0, c) * math.sqrt(d) / math.sqrt(1.0 + eps * d / (c * c))
        for round_a in (True, False):
            s_used = BF.round_to_bf16(s) if round_a else s
            if eps == 1e-30:
                assert s_used == math.copysign(16.0, c)      # exact: both modes coincide
            z = s_used * Wcol
            order = sorted(range(V), key=lambda v: (-z[v], v))[:k]
            lse = max(z) + LOG(math.fsum(math.exp(x - max(z)) for x in z))
            got = O.lens_project(to_bits(h), to_bits(np.ones(d)), W, eps, k, np.array([5]), round_a=round_a)
            assert list(got["topk_ids"][0]) == order
            np.testing.assert_allclose(got["topk_logits"][0], z[order], rtol=1e-13)
            assert abs(got["lse"][0] - lse) < 1e-12
            assert abs(got["target_logp"][0] - (z[5] - lse)) < 1e-12


def pin_zero_row(O):
    d, V, k = 32, 50, 7
    _, g, W, _ = rand_case(5, 1, d, V)
    out = O.lens_project(np.zeros((2, d), dtype=np.uint16), g, W, 1e-5, k, np.array([3, 49]))
    assert np.array_equal(out["topk_ids"], np.tile(np.arange(k), (2, 1)))
    np.testing.assert_allclose(out["topk_p"], 1.0 / V, rtol=1e-14)
    np.testing.assert_allclose(out["entropy"], LOG(V), rtol=1e-14)
    np.testing.assert_allclose(out["target_logp"], -LOG(V), rtol=1e-14)


def pin_eps_and_gamma(O):
    """A constant tiny row: the closed form shows where eps sits and that gamma multiplies."""
    d, V, k = 64, 20, 3
    rng = np.random.default_rng(11)
    W = to_bits(rng.standard_normal((V, d)))
    Wf = bits_to_float(W)
    c, eps = 2.0 ** -10, 1e-5
    h = to_bits(np.full((1, d), c))
    for gval in (1.0, 0.5):
        a1 = gval * c / math.sqrt(c * c + eps)          # mean of squares = c^2
        z = np.array([a1 * math.fsum(Wf[v]) for v in range(V)])
        order = sorted(range(V), key=lambda v: (-z[v], v))[:k]
        got = O.lens_project(h, to_bits(np.full(d, gval)), W, eps, k, None, round_a=False)
        assert list(got["topk_ids"][0]) == order
        np.testing.assert_allclose(got["topk_logits"][0], z[order], rtol=1e-12)
    # a per-channel gamma: only channel 0 kept
    gsel = np.zeros(d); gsel[0] = 2.0
    got = O.lens_project(h, to_bits(gsel), W, eps, k, None, round_a=False)
    z = 2.0 * c / math.sqrt(c * c + eps) * Wf[:, 0]
    np.testing.assert_allclose(got["topk_logits"][0], np.sort(z)[::-1][:k], rtol=1e-12)


def pin_scale_invariance(O):
    h, g, W, t = rand_case(13, 6, 32, 40)
    hf = bits_to_float(h)
    a = O.lens_project(h, g, W, 0.0, 5, t)
    b = O.lens_project(to_bits(hf * 8.0), g, W, 0.0, 5, t)       # exact power-of-two scaling
    assert np.array_equal(a["topk_ids"], b["topk_ids"])
    np.testing.assert_allclose(a["entropy"], b["entropy"], rtol=1e-13)
    np.testing.assert_allclose(a["target_logp"], b["target_logp"], rtol=1e-13)
    # with eps > 0 the change is bounded by eps * d / ||h||^2 (relative, on the normalised row)
    eps = 1e-3
    a = O.rmsnorm(h, g, eps, round_a=False)
    b = O.rmsnorm(to_bits(hf * 8.0), g, eps, round_a=False)
    bound = eps * 32 / np.sum(hf * hf, axis=1, keepdims=True)
    assert np.all(np.abs(a - b) <= np.abs(b) * bound)
    assert np.any(a != b)


def pin_library_routines(O):
    h, g, W, t = rand_case(17, 8, 48, 120)
    k = 10
    out = O.lens_project(h, g, W, 1e-5, k, t)
    hf, gf, Wf = bits_to_float(h), bits_to_float(g), bits_to_float(W)
    a = gf * hf / np.sqrt((hf * hf).mean(1, keepdims=True) + 1e-5)
    a = bits_to_float(to_bits(a))          # fp64 -> fp32 -> bf16 by torch; double rounding is negligible here
    z = torch.tensor(a) @ torch.tensor(Wf).T
    np.testing.assert_allclose(out["lse"], scipy.special.logsumexp(z.numpy(), axis=1), atol=1e-9)
    np.testing.assert_allclose(out["entropy"],
                               scipy.stats.entropy(scipy.special.softmax(z.numpy(), axis=1), axis=1), atol=1e-9)
    tv, ti = torch.topk(z, k, dim=1)
    assert np.array_equal(out["topk_ids"], ti.numpy())
    np.testing.assert_allclose(out["topk_p"], torch.softmax(z, 1).gather(1, ti).numpy(), atol=1e-10)
    np.testing.assert_allclose(out["target_logp"],
                               torch.log_softmax(z, 1)[torch.arange(8), torch.tensor(t)].numpy(), atol=1e-9)


def pin_permutation(O):
    """Channels permuted consistently in h, gamma and W change nothing; vocabulary rows permute the ids."""
    h, g, W, t = rand_case(19, 5, 24, 30)
    base = O.lens_project(h, g, W, 1e-5, 4, t, round_a=False)
    rng = np.random.default_rng(0)
    pc = rng.permutation(24)
    alt = O.lens_project(h[:, pc], g[pc], W[:, pc], 1e-5, 4, t, round_a=False)
    assert np.array_equal(base["topk_ids"], alt["topk_ids"])
    np.testing.assert_allclose(base["entropy"], alt["entropy"], rtol=1e-12)
    pv = rng.permutation(30)
    inv = np.argsort(pv)
    alt = O.lens_project(h, g, W[pv], 1e-5, 4, inv[t], round_a=False)
    assert np.array_equal(pv[alt["topk_ids"]], base["topk_ids"])
    np.testing.assert_allclose(base["target_logp"], alt["target_logp"], rtol=1e-12)


def pin_synthetic_entropy_band(O):
    """Gaussian W_out with std s: logits ~ N(0, s^2 |a|^2), so E[entropy] ~ log V - s^2 |a|^2 / 2."""
    rng = np.random.default_rng(23)
    d, V, R = 256, 4096, 16
    h = to_bits(rng.standard_normal((R, d)))
    g = to_bits(1.0 + 0.1 * rng.standard_normal(d))
    W = to_bits(0.02 * rng.standard_normal((V, d)))
    out = O.lens_project(h, g, W, 1e-5, 5, None)
    a = O.rmsnorm(h, g, 1e-5)
    var = 0.02 ** 2 * np.sum(a * a, axis=1)
    assert abs(np.mean(out["entropy"]) - np.mean(LOG(V) - var / 2)) < 0.01
    assert abs(np.mean(out["lse"]) - np.mean(LOG(V) + var / 2)) < 0.01


def pin_topk_renormalised(O):
    h, g, W, t = rand_case(29, 4, 16, 25)
    out = O.lens_project(h, g, W, 1e-5, 6, t)
    want = scipy.special.softmax(out["topk_logits"], axis=1)     # the paper's variant, Sec. 3.3
    np.testing.assert_allclose(O.topk_renormalised(out["topk_p"]), want, rtol=1e-12)


def pin_steer_vector(O):
    rng = np.random.default_rng(31)
    base = to_bits(rng.standard_normal((5, 12)))
    targ = to_bits(rng.standard_normal((7, 12)) + 1.0)
    v = O.steer_vector(base, targ)
    want = BF.steer_vector([list(r) for r in bits_to_float(base)], [list(r) for r in bits_to_float(targ)])
    np.testing.assert_allclose(v, want, rtol=1e-13)
    assert abs(np.sum(v * v) - 1.0) < 1e-13
    np.testing.assert_allclose(O.steer_vector(targ, base), -v, rtol=1e-13)
    raw = O.steer_vector(base, targ, normalize=False)
    np.testing.assert_allclose(raw, bits_to_float(targ).mean(0) - bits_to_float(base).mean(0), rtol=1e-13)
    assert np.dot(raw, v) > 0                                   # points from base to target
    # one matched pair: exactly Eq. (2)
    yp, ym = bits_to_float(targ[:1])[0], bits_to_float(base[:1])[0]
    np.testing.assert_allclose(O.steer_vector(base[:1], targ[:1]), (yp - ym) / np.linalg.norm(yp - ym), rtol=1e-13)
    assert np.array_equal(O.steer_vector(base, base), np.zeros(12))


def pin_steer_inject(O):
    h, g, W, t = rand_case(37, 6, 32, 60, scale=3.0)
    rng = np.random.default_rng(5)
    v = rng.standard_normal(32); v /= np.linalg.norm(v)
    # alpha = 0 is the identity on the bf16 normalised rows
    h0 = O.steer_inject(h, g, 1e-5, v, 0.0)
    assert np.array_equal(h0, O.f64_to_bf16_bits(O.rmsnorm(h, g, 1e-5, round_a=False)))
    a = O.lens_project(h0, None, W, 1e-5, 5, t)
    b = O.lens_project(h, g, W, 1e-5, 5, t)
    for key in ("topk_ids", "topk_p", "entropy", "target_logp"):
        assert np.array_equal(a[key], b[key])
    # Eq. (3): the injected rows are norm(h) + alpha v up to one bf16 rounding (rel. 2^-8)
    hf, gf = bits_to_float(h), bits_to_float(g)
    norm = gf * hf / np.sqrt((hf * hf).mean(1, keepdims=True) + 1e-5)
    for alpha in (-4.0, 1.5):
        got = bits_to_float(O.steer_inject(h, g, 1e-5, v, alpha))
        want = norm + alpha * v
        assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -8 + 1e-30)
    # logits move linearly in alpha along W v: the token whose row is argmax(W v) gains log-prob monotonically
    Wf = bits_to_float(W)
    tok = int(np.argmax(Wf @ v))
    lp = [O.lens_project(O.steer_inject(h, g, 1e-5, v, al), None, W, 1e-5, 5,
                         np.full(6, tok))["target_logp"] for al in (-4, -2, 0, 2, 4)]
    assert np.all(np.diff(np.array(lp), axis=0) > 0)


def pin_steer_sweep(O):
    """Several steering strengths at once: brute force on the steered rows, alpha = 0, and a direction along one channel."""
    h, g, W, t = rand_case(77, 3, 8, 13)
    rng = np.random.default_rng(5)
    v = rng.standard_normal(8).astype(np.float32)
    alphas = [-2.0, 0.0, 0.5, 3.0]
    got = O.steer_sweep(h, g, W, 1e-5, v, alphas, t)
    assert got["top1_ids"].shape == (4, 3)
    hf, gf, Wf = bits_to_float(h), bits_to_float(g), bits_to_float(W)
    for ai, al in enumerate(alphas):
        for r in range(3):
            ms = math.fsum(x * x for x in hf[r]) / 8
            a = [BF.round_to_bf16(gf[j] * hf[r][j] / math.sqrt(ms + 1e-5)) for j in range(8)]
            steered = [a[j] + al * float(v[j]) for j in range(8)]
            want = BF.project_row(steered, None, [list(w) for w in Wf], 1e-5, 1, int(t[r]))
            assert got["top1_ids"][ai, r] == want["ids"][0]
            assert abs(got["top1_p"][ai, r] - want["p"][0]) < 1e-12
            assert abs(got["entropy"][ai, r] - want["entropy"]) < 1e-12
            assert abs(got["target_logp"][ai, r] - want["target_logp"]) < 1e-12
    # the k most likely tokens per alpha (the paper's figures list three per cell): brute force again, every rank
    got3 = O.steer_sweep(h, g, W, 1e-5, v, alphas, t, k=3)
    assert got3["topk_ids"].shape == (4, 3, 3) and got3["topk_p"].shape == (4, 3, 3)
    for ai, al in enumerate(alphas):
        for r in range(3):
            ms = math.fsum(x * x for x in hf[r]) / 8
            a = [BF.round_to_bf16(gf[j] * hf[r][j] / math.sqrt(ms + 1e-5)) for j in range(8)]
            want = BF.project_row([a[j] + al * float(v[j]) for j in range(8)], None, [list(w) for w in Wf], 1e-5, 3, int(t[r]))
            assert list(got3["topk_ids"][ai, r]) == want["ids"]
            assert max(abs(got3["topk_p"][ai, r, i] - want["p"][i]) for i in range(3)) < 1e-12
    assert np.array_equal(got3["top1_ids"], got["top1_ids"]) and np.array_equal(got3["topk_ids"][:, :, 0], got["top1_ids"])
    np.testing.assert_array_equal(got3["entropy"], got["entropy"])           # the list length changes nothing else
    assert np.all(np.diff(got3["topk_p"], axis=2) <= 0)
    base3 = O.lens_project(h, g, W, 1e-5, 3, t)
    assert np.array_equal(got3["topk_ids"][1], base3["topk_ids"])              # alpha = 0: the plain projection's list
    np.testing.assert_allclose(got3["topk_p"][1], base3["topk_p"], rtol=1e-13)
    # alpha = 0 is the plain projection
    base = O.lens_project(h, g, W, 1e-5, 1, t)
    assert np.array_equal(got["top1_ids"][1], base["topk_ids"][:, 0])
    np.testing.assert_allclose(got["entropy"][1], base["entropy"], rtol=1e-13)
    np.testing.assert_allclose(got["target_logp"][1], base["target_logp"], rtol=1e-13)
    # along channel j the shift of logit id is alpha * W[id, j]: a large alpha picks the largest / smallest entry
    e = np.zeros(8, np.float32); e[3] = 1.0
    far = O.steer_sweep(h, g, W, 1e-5, e, [1e4, -1e4], None)
    assert np.all(far["top1_ids"][0] == int(np.argmax(Wf[:, 3]))) and np.all(far["top1_ids"][1] == int(np.argmin(Wf[:, 3])))
    # rows that are already normalised are used as they are
    a_bits = O.f64_to_bf16_bits(O.rmsnorm(h, g, 1e-5))
    again = O.steer_sweep(a_bits, None, W, 1e-5, v, alphas, t)
    np.testing.assert_allclose(again["entropy"], got["entropy"], rtol=1e-13)


def pin_steer_inject_raw(O):
    """In-model injection: the plain equation without clipping, a hand-computed clipped row, and the clipping bound."""
    rng = np.random.default_rng(11)
    h = to_bits(rng.standard_normal((5, 16)) * 3)
    hf = bits_to_float(h)
    v = rng.standard_normal(16); v /= np.linalg.norm(v)
    # no clipping: h + alpha * scale * v, one rounding (brute force with the pure-Python rounding)
    got = bits_to_float(O.steer_inject_raw(h, v, 1.5, 2.0, 0.0))
    for r in range(5):
        want = [BF.round_to_bf16(float(hf[r, j]) + 3.0 * float(v[j])) for j in range(16)]
        assert list(got[r]) == want
    # hand-made row of length 5, unit direction along a free channel: alpha 10 clipped to 0.2 * 5 = 1
    row = np.zeros((1, 8)); row[0, 0], row[0, 1] = 3.0, 4.0
    e = np.zeros(8); e[2] = 1.0
    out = bits_to_float(O.steer_inject_raw(to_bits(row), e, 10.0, 1.0, 0.2))
    assert list(out[0]) == [3.0, 4.0, 1.0, 0, 0, 0, 0, 0]
    out = bits_to_float(O.steer_inject_raw(to_bits(row), e, -10.0, 1.0, 0.2))
    assert out[0, 2] == -1.0                                   # the sign survives the clipping
    out = bits_to_float(O.steer_inject_raw(to_bits(row), e, 0.5, 1.0, 0.2))
    assert out[0, 2] == 0.5                                    # below the cap: untouched
    out = bits_to_float(O.steer_inject_raw(to_bits(row), e, 0.5, 4.0, 0.2))
    assert out[0, 2] == 1.0                                    # the layer's scale counts before the clipping
    # the shift never exceeds clip_ratio * ||h|| (plus the output rounding), and reaches it when clipped
    big = bits_to_float(O.steer_inject_raw(h, v, 100.0, 1.0, 0.25))
    shift = np.linalg.norm(big - hf, axis=1)
    cap = 0.25 * np.linalg.norm(hf, axis=1)
    assert np.all(shift <= cap * 1.01) and np.all(shift >= cap * 0.99)


def pin_concat_trajectories(O):
    """Appending slices step by step gives the same store as writing every token where it belongs."""
    rng = np.random.default_rng(3)
    L, C, d = 3, 2, 8
    steps = [rng.integers(0, 65536, size=(L * C, n, d)).astype(np.uint16) for n in (5, 1, 1, 3, 1)]
    H = O.concat_trajectories(steps, L, C)
    assert H.shape == (L, C, 11, d) and H.dtype == np.uint16
    t = 0
    for sl in steps:
        for i in range(sl.shape[1]):
            for l in range(L):
                for c in range(C):
                    assert np.array_equal(H[l, c, t], sl[l * C + c, i])
            t += 1


PINS = [pin_bf16_widen, pin_bf16_round, pin_brute_force, pin_bias, pin_invariants, pin_one_hot, pin_zero_row,
        pin_eps_and_gamma, pin_scale_invariance, pin_library_routines, pin_permutation,
        pin_synthetic_entropy_band, pin_topk_renormalised, pin_steer_vector, pin_steer_inject, pin_steer_sweep, pin_steer_inject_raw,
        pin_concat_trajectories]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_pin(pin):
    pin(ORACLE)


# ----------------------------------------------------------------------------
# planted mistakes: each must be caught by at least one pin
# ----------------------------------------------------------------------------
@contextlib.contextmanager
def patched(**repl):
    saved = {k: getattr(ORACLE, k) for k in repl}
    try:
        for k, f in repl.items():
            setattr(ORACLE, k, f)
        yield
    finally:
        for k, f in saved.items():
            setattr(ORACLE, k, f)


_real = {n: getattr(ORACLE, n) for n in ORACLE.__all__}


def _rmsnorm_variant(kind):
    def f(hidden_bits, gamma_bits, eps, round_a=True):
        h = _real["bf16_bits_to_f64"](hidden_bits)
        if gamma_bits is None:
            return h
        g = _real["bf16_bits_to_f64"](gamma_bits)
        ms = np.mean(h * h, axis=-1, keepdims=True)
        if kind == "no_eps":
            a = g * h / np.sqrt(ms)
        elif kind == "eps_outside":
            a = g * h / (np.sqrt(ms) + eps)
        elif kind == "layernorm":
            hc = h - h.mean(-1, keepdims=True)
            a = g * hc / np.sqrt(np.mean(hc * hc, -1, keepdims=True) + eps)
        elif kind == "no_gamma":
            a = h / np.sqrt(ms + eps)
        elif kind == "sum_not_mean":
            a = g * h / np.sqrt(ms * h.shape[-1] + eps)
        elif kind == "round_via_fp32":
            a = g * h / np.sqrt(ms + eps)
        if round_a:
            a = _real["bf16_bits_to_f64"](_real["f64_to_bf16_bits"](a))
        return a
    return f


def _round_via_fp32(x):
    t = torch.tensor(np.asarray(x, dtype=np.float64)).to(torch.float32).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def _summaries_variant(kind):
    def f(z, k, target_ids=None):
        out = dict(_real["softmax_summaries"](z, k, target_ids))
        if kind == "smallest_k":
            o2 = _real["softmax_summaries"](-z, k, target_ids)
            out["topk_ids"] = o2["topk_ids"]
            out["topk_logits"] = -o2["topk_logits"]
            out["topk_p"] = np.exp(out["topk_logits"] - out["lse"][:, None])
        elif kind == "entropy_drops_lse":
            p = np.exp(z - out["lse"][:, None])
            out["entropy"] = -np.sum(p * z, axis=1)
        elif kind == "ties_descending_id":
            order = np.argsort(-z[:, ::-1], axis=1, kind="stable")
            ids = (z.shape[1] - 1 - order)[:, :k]
            out["topk_ids"] = ids.astype(np.int32)
        elif kind == "topk_only_softmax":
            out["topk_p"] = out["topk_p"] / out["topk_p"].sum(1, keepdims=True)
        elif kind == "unshifted_target":
            if target_ids is not None:
                out["target_logp"] = out["target_logp"] + out["lse"]
        return out
    return f


def _logits_transposed(a, w_bits, slab=8192, bias=None):
    w = _real["bf16_bits_to_f64"](w_bits)
    return a @ w if w.shape[0] == w.shape[1] else _real["full_logits"](a, w_bits, bias=bias)


def _logits_bias_dropped(a, w_bits, slab=8192, bias=None):
    return _real["full_logits"](a, w_bits)


def _logits_bias_subtracted(a, w_bits, slab=8192, bias=None):
    return _real["full_logits"](a, w_bits, bias=None if bias is None else -np.asarray(bias))


def _steer_variant(kind):
    def f(base_bits, target_bits, normalize=True):
        if kind == "sign":
            return _real["steer_vector"](target_bits, base_bits, normalize)
        if kind == "never_normalised":
            return _real["steer_vector"](base_bits, target_bits, False)
        if kind == "normalise_rows_first":
            b = _real["bf16_bits_to_f64"](base_bits); t = _real["bf16_bits_to_f64"](target_bits)
            b = b / np.linalg.norm(b, axis=1, keepdims=True)
            t = t / np.linalg.norm(t, axis=1, keepdims=True)
            diff = t.mean(0) - b.mean(0)
            return diff / np.linalg.norm(diff) if normalize and np.linalg.norm(diff) > 0 else diff
    return f


def _inject_variant(kind):
    def f(hidden_bits, gamma_bits, eps, v, alpha):
        if kind == "pre_norm":       # adds alpha v before the normalisation
            h = _real["bf16_bits_to_f64"](hidden_bits) + alpha * np.asarray(v)[None, :]
            g = _real["bf16_bits_to_f64"](gamma_bits)
            a = g * h / np.sqrt(np.mean(h * h, -1, keepdims=True) + eps)
            return _real["f64_to_bf16_bits"](a)
        if kind == "minus":
            return _real["steer_inject"](hidden_bits, gamma_bits, eps, v, -alpha)
    return f


def _sweep_variant(kind):
    def f(hidden_bits, gamma_bits, w_bits, eps, v, alphas, target_ids=None, round_a=True, k=1):
        if kind == "minus":
            return _real["steer_sweep"](hidden_bits, gamma_bits, w_bits, eps, v, [-x for x in alphas], target_ids, round_a, k)
        if kind == "rounds_steered_rows":   # what inject + project does, not what the sweep is defined as
            outs = []
            for al in alphas:
                if gamma_bits is None:
                    a = _real["bf16_bits_to_f64"](hidden_bits) + al * np.asarray(v, np.float64)[None, :]
                    bits = _real["f64_to_bf16_bits"](a)
                else:
                    a = _real["rmsnorm"](hidden_bits, gamma_bits, eps, round_a=True) + al * np.asarray(v, np.float64)[None, :]
                    bits = _real["f64_to_bf16_bits"](a)
                outs.append(_real["lens_project"](bits, None, w_bits, eps, k, target_ids))
            return {"top1_ids": np.stack([o["topk_ids"][:, 0] for o in outs]), "top1_p": np.stack([o["topk_p"][:, 0] for o in outs]),
                    "topk_ids": np.stack([o["topk_ids"] for o in outs]), "topk_p": np.stack([o["topk_p"] for o in outs]),
                    "topk_logits": np.stack([o["topk_logits"] for o in outs]),
                    "target_logp": np.stack([o["target_logp"] for o in outs]), "entropy": np.stack([o["entropy"] for o in outs])}
        if kind == "unnormalised_rows":     # steering added to the raw hidden state
            return _real["steer_sweep"](hidden_bits, None, w_bits, eps, v, alphas, target_ids, round_a, k)
        if kind == "lists_of_unsteered_logits":   # statistics per alpha, but every alpha lists the tokens of alpha = 0
            out = _real["steer_sweep"](hidden_bits, gamma_bits, w_bits, eps, v, alphas, target_ids, round_a, k)
            zero = _real["steer_sweep"](hidden_bits, gamma_bits, w_bits, eps, v, [0.0], target_ids, round_a, k)
            for key in ("topk_ids", "topk_p", "topk_logits"):
                out[key] = np.repeat(zero[key], len(alphas), axis=0)
            return out
    return f


def _inject_raw_variant(kind):
    def f(hidden_bits, v, alpha, layer_scale=1.0, clip_ratio=0.0):
        h = _real["bf16_bits_to_f64"](hidden_bits)
        s = alpha * layer_scale
        if kind == "scale_after_clip":
            cap = clip_ratio * np.sqrt(np.sum(h * h, -1, keepdims=True)) if clip_ratio > 0 else np.inf
            beta = np.sign(alpha) * np.minimum(abs(alpha), cap) * layer_scale
        elif kind == "clip_to_rms":
            cap = clip_ratio * np.sqrt(np.mean(h * h, -1, keepdims=True)) if clip_ratio > 0 else np.inf
            beta = np.sign(s) * np.minimum(abs(s), cap)
        elif kind == "sign_lost":
            cap = clip_ratio * np.sqrt(np.sum(h * h, -1, keepdims=True)) if clip_ratio > 0 else np.inf
            beta = np.minimum(abs(s), cap) * np.ones((h.shape[0], 1))
        return _real["f64_to_bf16_bits"](h + beta * np.asarray(v, np.float64)[None, :])
    return f


def _concat_variant(kind):
    def f(step_slices, L, C):
        full = np.concatenate([np.asarray(x) for x in step_slices], axis=1)
        if kind == "type_major":      # (type, layer) instead of (layer, type)
            return full.reshape(C, L, full.shape[1], full.shape[2]).transpose(1, 0, 2, 3)
    return f


MUTANTS = {
    "rmsnorm_no_eps": dict(rmsnorm=_rmsnorm_variant("no_eps")),
    "rmsnorm_eps_outside_sqrt": dict(rmsnorm=_rmsnorm_variant("eps_outside")),
    "rmsnorm_is_layernorm": dict(rmsnorm=_rmsnorm_variant("layernorm")),
    "rmsnorm_no_gamma": dict(rmsnorm=_rmsnorm_variant("no_gamma")),
    "rmsnorm_sum_not_mean": dict(rmsnorm=_rmsnorm_variant("sum_not_mean")),
    "bf16_round_via_fp32": dict(f64_to_bf16_bits=_round_via_fp32),
    "topk_smallest": dict(softmax_summaries=_summaries_variant("smallest_k")),
    "entropy_drops_lse": dict(softmax_summaries=_summaries_variant("entropy_drops_lse")),
    "ties_descending_id": dict(softmax_summaries=_summaries_variant("ties_descending_id")),
    "p_is_topk_only_softmax": dict(softmax_summaries=_summaries_variant("topk_only_softmax")),
    "target_logit_not_logp": dict(softmax_summaries=_summaries_variant("unshifted_target")),
    "logits_transposed": dict(full_logits=_logits_transposed),
    "bias_dropped": dict(full_logits=_logits_bias_dropped),
    "bias_subtracted": dict(full_logits=_logits_bias_subtracted),
    "steer_sign": dict(steer_vector=_steer_variant("sign")),
    "steer_never_normalised": dict(steer_vector=_steer_variant("never_normalised")),
    "steer_normalise_rows_first": dict(steer_vector=_steer_variant("normalise_rows_first")),
    "inject_pre_norm": dict(steer_inject=_inject_variant("pre_norm")),
    "inject_minus": dict(steer_inject=_inject_variant("minus")),
    "sweep_minus": dict(steer_sweep=_sweep_variant("minus")),
    "sweep_rounds_steered_rows": dict(steer_sweep=_sweep_variant("rounds_steered_rows")),
    "sweep_unnormalised_rows": dict(steer_sweep=_sweep_variant("unnormalised_rows")),
    "sweep_lists_of_unsteered_logits": dict(steer_sweep=_sweep_variant("lists_of_unsteered_logits")),
    "inject_raw_scale_after_clip": dict(steer_inject_raw=_inject_raw_variant("scale_after_clip")),
    "inject_raw_clip_to_rms": dict(steer_inject_raw=_inject_raw_variant("clip_to_rms")),
    "inject_raw_sign_lost": dict(steer_inject_raw=_inject_raw_variant("sign_lost")),
    "concat_type_major": dict(concat_trajectories=_concat_variant("type_major")),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    failed = []
    with patched(**MUTANTS[name]):
        for pin in PINS:
            try:
                pin(ORACLE)
            except Exception:            # an assertion, or a shape error from the mistake
                failed.append(pin.__name__)
    assert failed, f"no pin notices the planted mistake {name!r}"
