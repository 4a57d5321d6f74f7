"""Steering sweep (paper Sec. 3.4, Eq. 3 read out through the lens for several alpha in one pass)
against the CPU oracle, on a real MI355X."""
import sys

import numpy as np
import pytest
import torch

import oracle.lens_oracle as O
from paper_2604_06483_amd import binding as LL
from paper_2604_06483_amd import workloads as WL
from tests import parity as P
from tests.conftest import say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ALPHAS9 = [-4.0, -3.0, -2.0, -1.0, 0.0, 1.0, 2.0, 3.0, 4.0]



def direction(d, seed=3):
    g = torch.Generator(device=DEV).manual_seed(seed)
    v = torch.randn((d,), generator=g, device=DEV)
    return v / v.norm()


def compare_sweep(got, want, rows, label, inputs):
    """got: tuple of GPU tensors [A, N] or [A, N, k]; want: oracle dict for the sampled rows (computed with the same
    k); inputs = (hidden_bits of those rows, gamma_bits or None, w_bits, eps, v, alphas): where an id differs from
    the oracle's, the oracle's own logit of the library's id is formed from them (Eq. 3 through the lens, one
    entry: W_U[id] . (a + alpha v)) and must lie within the tie band of the oracle's logit at that rank."""
    ids, p, logp, ent = (None if t is None else t.cpu().numpy()[:, rows] for t in got)
    if ids.ndim == 2:
        ids, p = ids[:, :, None], p[:, :, None]
    assert np.abs(ent - want["entropy"]).max() <= P.TOL_ENT, f"{label}: entropy off by {np.abs(ent - want['entropy']).max():.3e}"
    if logp is not None:
        nan_w = np.isnan(want["target_logp"])
        assert np.array_equal(np.isnan(logp), nan_w), f"{label}: NaN pattern"
        assert np.abs(logp[~nan_w] - want["target_logp"][~nan_w]).max(initial=0.0) <= P.TOL_LOGP, f"{label}: target_logp"
    k = ids.shape[2]
    want_p, want_ids, want_z = want["topk_p"][:, :, :k], want["topk_ids"][:, :, :k], want["topk_logits"][:, :, :k]
    assert np.abs(p - want_p).max() <= P.TOL_P, f"{label}: listed probability off"
    big = want_p > P.P_FLOOR
    assert np.abs(np.log(p[big].astype(np.float64)) - np.log(want_p[big])).max(initial=0.0) <= P.TOL_LOG_P, f"{label}: log p"
    V = inputs[2].shape[0]
    assert ids.min() >= 0 and ids.max() < V, f"{label}: id out of range"
    if k > 1:
        srt = np.sort(ids, axis=2)
        assert np.all(srt[:, :, 1:] != srt[:, :, :-1]), f"{label}: duplicate ids in a list"
    hb, gb, wb, eps, v, alphas = inputs
    a_rows = O.rmsnorm(hb, gb, eps) if gb is not None else O.bf16_bits_to_f64(hb)
    vv = np.asarray(v, dtype=np.float64)
    mism = np.argwhere(ids != want_ids)
    for ai, r, j in mism:
        w_row = O.bf16_bits_to_f64(wb[int(ids[ai, r, j])])
        z_lib_choice = float(w_row @ (a_rows[r] + float(alphas[ai]) * vv))
        assert abs(z_lib_choice - want_z[ai, r, j]) < P.TIE_BAND, (
            f"{label}: alpha {alphas[ai]} row {rows[r]} rank {j}: id {ids[ai, r, j]} (oracle logit {z_lib_choice:.6f}) is not a "
            f"near-tie of oracle id {want_ids[ai, r, j]} (logit {want_z[ai, r, j]:.6f})")
    return len(mism), ids.size


@pytest.mark.parametrize("N,d,V,n_alpha,gamma", [
    (64, 256, 4096, 9, True),        # the tiny config's shape
    (300, 512, 5000, 9, True),       # ragged rows and vocabulary, two row blocks
    (257, 128, 777, 3, True),        # few alphas, odd vocabulary
    (520, 1024, 33000, 5, False),    # rows already normalised, many tiles per split
    (40, 64, 300, 1, True),          # a single alpha, one K step
    (9000, 128, 1000, 2, True),      # two row passes: the second starts at row 8192 of every output
    (200, 328, 1000, 9, True),       # d not a multiple of 64: the register-staged kernel, norm inside its A-tile load
    (130, 72, 600, 4, False),        # the same with rows that are already normalised
    (40, 40960, 300, 2, True),       # the largest hidden size admitted (the direction fills the LDS)
])
def test_sweep_matches_oracle(N, d, V, n_alpha, gamma):
    say(f"sweep N={N} d={d} V={V} A={n_alpha} gamma={gamma}")
    cfg = WL.LensConfig("sw", L=1, T=N, d=d, V=V, k=1, n_outliers=min(4, d // 16), outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=21)
    v = direction(d)
    alphas = ALPHAS9[:n_alpha] if n_alpha != 5 else [-4.0, -0.5, 0.0, 1.25, 4.0]
    hidden = w.hidden.reshape(N, d)
    if not gamma:
        hidden = LL.ll_steer_inject(hidden, w.gamma, cfg.eps, v, 0.0)      # bf16(RMSNorm(h))
    tgt = w.target_ids.clone()
    tgt[0] = -5
    tgt[N - 1] = V                                                           # outside the vocabulary: NaN
    got = LL.ll_steer_sweep(hidden, w.gamma if gamma else None, w.W_U, cfg.eps, v, alphas, tgt)
    torch.cuda.synchronize()
    rows = np.arange(N)
    inputs = (WL.bf16_bits(hidden), WL.bf16_bits(w.gamma) if gamma else None, WL.bf16_bits(w.W_U), cfg.eps, v.cpu().numpy(),
              alphas)
    want = O.steer_sweep(*inputs, tgt.cpu().numpy())
    mism, total = compare_sweep(got, want, rows, f"N={N} d={d} V={V}", inputs)
    say(f"sweep N={N} d={d} V={V}: {mism} of {total} arg max ids differ from the oracle's, each a near-tie")
    # without targets
    got2 = LL.ll_steer_sweep(hidden, w.gamma if gamma else None, w.W_U, cfg.eps, v, alphas, None)
    torch.cuda.synchronize()
    assert got2[2] is None and torch.equal(got2[0], got[0]) and torch.equal(got2[3], got[3])


@pytest.mark.parametrize("N,d,V,n_alpha,k,gamma", [
    (300, 512, 5000, 9, 3, True),     # nine alphas, two passes of the kernel (5 + 4), two row blocks
    (257, 128, 777, 5, 4, True),      # the longest list, ragged vocabulary
    (64, 256, 4096, 4, 2, False),     # one pass; rows already normalised
    (200, 328, 1000, 9, 3, True),     # d not a multiple of 64: the register-staged kernel
    (9000, 128, 1000, 6, 2, True),    # two row passes
    (33, 64, 3, 2, 3, True),          # k = V: every token listed
])
def test_sweep_with_lists_matches_oracle(N, d, V, n_alpha, k, gamma):
    say(f"sweep with lists N={N} d={d} V={V} A={n_alpha} k={k} gamma={gamma}")
    cfg = WL.LensConfig("swk", L=1, T=N, d=d, V=V, k=k, n_outliers=min(4, d // 16), outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=22)
    v = direction(d)
    alphas = ALPHAS9[:n_alpha] if n_alpha != 5 else [-4.0, -0.5, 0.0, 1.25, 4.0]
    hidden = w.hidden.reshape(N, d)
    if not gamma:
        hidden = LL.ll_steer_inject(hidden, w.gamma, cfg.eps, v, 0.0)
    tgt = w.target_ids.clone()
    tgt[0] = -5
    got = LL.ll_steer_sweep(hidden, w.gamma if gamma else None, w.W_U, cfg.eps, v, alphas, tgt, k=k)
    torch.cuda.synchronize()
    assert tuple(got[0].shape) == (n_alpha, N, k) and tuple(got[3].shape) == (n_alpha, N)
    inputs = (WL.bf16_bits(hidden), WL.bf16_bits(w.gamma) if gamma else None, WL.bf16_bits(w.W_U), cfg.eps, v.cpu().numpy(),
              alphas)
    want = O.steer_sweep(*inputs, tgt.cpu().numpy(), k=k)
    mism, total = compare_sweep(got, want, np.arange(N), f"lists N={N} d={d} V={V} k={k}", inputs)
    say(f"sweep with lists N={N} d={d} V={V} k={k}: {mism} of {total} listed ids differ from the oracle's, each a near-tie")
    # the plain sweep gives the head of every list and the same statistics
    one = LL.ll_steer_sweep(hidden, w.gamma if gamma else None, w.W_U, cfg.eps, v, alphas, tgt)
    torch.cuda.synchronize()
    assert torch.equal(one[0], got[0][:, :, 0])
    assert (one[3] - got[3]).abs().max().item() < 1e-5 and (one[1] - got[1][:, :, 0]).abs().max().item() < 1e-6


def test_sweep_alpha_zero_equals_projection():
    say("sweep alpha=0 vs ll_project")
    cfg = WL.LensConfig("sw0", L=2, T=300, d=512, V=9000, k=1, n_outliers=4, outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=5)
    v = direction(cfg.d)
    ids, p, logp, ent = LL.ll_steer_sweep(w.hidden, w.gamma, w.W_U, cfg.eps, v, [0.0, 2.0], w.target_ids)
    pid, pp, plogp, pent = LL.ll_project(w.hidden, w.gamma, w.W_U, cfg.eps, 1, w.target_ids)
    torch.cuda.synchronize()
    # same operands, same accumulation order: only the final fp32 arithmetic of the merge differs
    assert torch.equal(ids[0], pid[:, 0])
    assert (ent[0] - pent).abs().max().item() < 1e-5
    assert (logp[0] - plogp).abs().max().item() < 1e-5
    assert (p[0] - pp[:, 0]).abs().max().item() < 1e-6


def test_sweep_close_to_inject_then_project():
    """The sweep leaves the steered row unrounded; inject + project rounds it to bf16 first.  The two
    agree to what that rounding moves a logit (reported by the oracle's two modes)."""
    say("sweep vs inject+project")
    cfg = WL.CONFIGS["tiny"]
    w = WL.make_workload(cfg, DEV)
    N = cfg.L * cfg.T
    v = direction(cfg.d)
    alphas = [-4.0, 0.0, 4.0]
    sw = LL.ll_steer_sweep(w.hidden, w.gamma, w.W_U, cfg.eps, v, alphas, w.target_ids)
    for ai, al in enumerate(alphas):
        steered = LL.ll_steer_inject(w.hidden, w.gamma, cfg.eps, v, al)
        ids, p, logp, ent = LL.ll_project(steered, None, w.W_U, cfg.eps, 1, w.target_ids)
        torch.cuda.synchronize()
        assert (sw[3][ai] - ent).abs().max().item() < 2e-2
        assert (sw[2][ai] - logp).abs().max().item() < 5e-2


@pytest.mark.parametrize("name", ["llama31-8b"])
def test_sweep_full_size_layer(name):
    """The steering workload at its real shape: the 1500 rows of the middle layer, nine alphas,
    oracle on a sample of rows."""
    cfg = WL.CONFIGS[name]
    say(f"sweep full size {name}")
    w = WL.make_workload(cfg, DEV)
    base, target, layer = WL.make_steer_rows(cfg, w.outlier_idx, DEV)
    v = LL.ll_steer_vector(base, target, True)
    rows_h = w.hidden.reshape(cfg.L, cfg.T, cfg.d)[layer].contiguous()
    tgt = w.target_ids.reshape(cfg.L, cfg.T)[layer].contiguous()
    got = LL.ll_steer_sweep(rows_h, w.gamma, w.W_U, cfg.eps, v, ALPHAS9, tgt)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, cfg.T - 1, 255, 256, 1279, 1280], np.random.default_rng(0).integers(0, cfg.T, 26)]))
    inputs = (WL.bf16_bits(rows_h)[rows], WL.bf16_bits(w.gamma), WL.bf16_bits(w.W_U), cfg.eps, v.cpu().numpy(), ALPHAS9)
    want = O.steer_sweep(*inputs, tgt.cpu().numpy()[rows], k=3)
    mism, total = compare_sweep(got, want, rows, name, inputs)
    say(f"sweep {name}: {mism} of {total} arg max ids differ from the oracle's, each a near-tie")
    # the same rows with the three most likely tokens per alpha (the paper's figures list k = 3): three passes over W_U
    got3 = LL.ll_steer_sweep(rows_h, w.gamma, w.W_U, cfg.eps, v, ALPHAS9, tgt, k=3)
    torch.cuda.synchronize()
    mism, total = compare_sweep(got3, want, rows, name + " k=3", inputs)
    say(f"sweep {name} k=3: {mism} of {total} listed ids differ from the oracle's, each a near-tie")
    assert torch.equal(got3[0][:, :, 0], got[0]) and torch.equal(got3[3], got[3])
    ent = got[3].cpu().numpy()
    assert np.all(np.isfinite(ent)) and ent.min() >= -1e-4 and ent.max() <= np.log(cfg.V) + 1e-4
