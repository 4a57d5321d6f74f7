"""Parity of the HIP library (through the C ABI) with the CPU oracle, on a real MI355X."""
import math
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



STAGED = False      # set per case: the register-staged kernel (norm inside its A-tile load) instead of the default one


@pytest.fixture(params=[2, 1], ids=["dma-panel", "fused-norm"], autouse=True)
def gemm_path(request):
    """Every case runs on both projection kernels (2: the default; 1: LL_FLAG_REGISTER_STAGED on every call)."""
    global STAGED
    STAGED = request.param == 1
    yield request.param
    STAGED = False


def project(*args, **kw):
    """LL.ll_project on the kernel the case is parametrised with."""
    if STAGED and not kw.get("timed"):
        kw["register_staged"] = True
    return LL.ll_project(*args, **kw)


def run_project(w, k=None, gamma="w", target=True):
    cfg = w.cfg
    res = project(w.hidden, w.gamma if gamma == "w" else gamma, w.W_U, cfg.eps, k or cfg.k,
                        w.target_ids if target else None)
    torch.cuda.synchronize()
    return P.to_numpy(res, has_target=target)


def oracle_for(w, rows, k=None, gamma="w"):
    cfg = w.cfg
    hb = WL.bf16_bits(w.hidden.reshape(-1, cfg.d)[torch.as_tensor(rows, device=w.hidden.device)])
    gb = WL.bf16_bits(w.gamma) if gamma == "w" else None
    wb = WL.bf16_bits(w.W_U)
    t = w.target_ids.cpu().numpy()[rows]
    return P.oracle_rows(hb, gb, wb, cfg.eps, k or cfg.k, t)


# ------------------------------------------------------------------------------------------
# small cases, every row checked: several tiles, ragged tails in N, d and V
# ------------------------------------------------------------------------------------------
def test_tiny_config_all_rows():
    say("tiny config")
    w = WL.make_workload("tiny", DEV)
    got = run_project(w)
    ref = oracle_for(w, np.arange(w.cfg.N))
    rep = P.compare(got, ref, w.cfg.k, label="tiny")
    P.check_invariants(got, w.cfg.V, w.cfg.k, label="tiny")
    say(f"tiny: {rep}")


RAGGED = [
    # name,            L,  T,   d,    V,   k, outliers
    ("tails",          3, 100,  328, 1000,  7, 2),      # N=300: 2 row blocks; d not a multiple of 64; V: 4 tiles, last partial
    ("one-row",        1,   1,   64,  300,  3, 0),
    ("tiny-vocab",     2,  33,  128,  100, 32, 0),      # V < one tile, k = LL_KMAX
    ("k-equals-V",     1,  20,   72,   24, 24, 0),
    ("k1-d8",          2,  70,    8,  513,  1, 0),      # smallest d, V = 2 tiles + 1
    ("many-blocks",    5, 300,  192, 2048, 10, 4),      # N=1500: 6 row blocks, 8 tiles
    ("wide-d",         1,  96, 1096,  777, 20, 0),
    # d a multiple of 64: these reach the direct-to-LDS kernel
    ("lds-ragged",     3, 171,  256, 3333, 12, 2),      # N=513: 3 row blocks, the last with one row; 14 tiles, last partial
    ("lds-k32",        2, 150,  320, 5000, 32, 0),      # 5 K stages, longest top-k list
    ("lds-one-stage",  1, 300,   64, 1500,  5, 0),      # a single K stage per tile
    ("lds-79-splits",  1,  64,  128, 20000, 20, 0),     # one row block: one vocabulary split per tile, four lists per merging lane
    ("lds-256-splits", 1,  81,  128, 70000, 20, 2),     # a decoding step's rows: 274 tiles over 256 splits
    ("lds-256-k32",    1,  40,   64, 70000, 32, 0),     # the same with the longest lists: 64 KB of them per row in the merge
    ("lds-128-splits", 2, 200,  192, 40000, 10, 2),     # two row blocks (the second ragged): 128 splits each
    ("lds-85-splits",  3, 250,   64, 30000,  4, 0),     # three row blocks: 85 splits, the last merging lane with one list
    ("lds-long-k",     1, 300, 16384, 1000, 10, 4),     # twice the largest paper-shaped hidden size: 256 K stages per tile
]


@pytest.mark.parametrize("case", RAGGED, ids=[c[0] for c in RAGGED])
def test_ragged_shapes_all_rows(case):
    name, L, T, d, V, k, n_out = case
    say(f"ragged {name}: N={L*T} d={d} V={V} k={k}")
    cfg = WL.LensConfig(name, L=L, T=T, d=d, V=V, k=k, n_outliers=n_out, outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=3)
    got = run_project(w)
    ref = oracle_for(w, np.arange(cfg.N))
    rep = P.compare(got, ref, k, label=name)
    P.check_invariants(got, V, k, label=name)
    say(f"{name}: {rep}")


def random_shapes(n, seed):
    """Seeded shapes over the whole ragged range: both kernels' d classes, one to three row blocks (every
    split count from 1 to 256), k from 1 to the maximum."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        d = int(rng.choice([8 * int(rng.integers(1, 130)), 64 * int(rng.integers(1, 17))]))
        N = int(rng.choice([int(rng.integers(1, 64)), int(rng.integers(64, 257)), int(rng.integers(257, 700))]))
        V = int(rng.choice([int(rng.integers(33, 600)), int(rng.integers(600, 9000)), int(rng.integers(9000, 70000))]))
        k = int(rng.choice([1, int(rng.integers(2, 13)), int(rng.integers(13, 33))]))
        if N * V * d > 6e9:          # keep the oracle's contraction to a few seconds per case
            V = max(33, int(6e9 / (N * d)))
        out.append((f"r{i}", N, d, V, min(k, V), int(rng.integers(0, 3))))
    return out


RANDOM = random_shapes(16, seed=20260406)


@pytest.mark.parametrize("case", RANDOM, ids=[f"{c[0]}-N{c[1]}-d{c[2]}-V{c[3]}-k{c[4]}" for c in RANDOM])
def test_random_shapes_all_rows(case):
    name, N, d, V, k, n_out = case
    say(f"random {name}: N={N} d={d} V={V} k={k} outliers={n_out}")
    cfg = WL.LensConfig(name, L=1, T=N, d=d, V=V, k=k, n_outliers=min(n_out, d), outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=11)
    got = run_project(w)
    ref = oracle_for(w, np.arange(cfg.N))
    rep = P.compare(got, ref, k, label=name)
    P.check_invariants(got, V, k, label=name)
    say(f"{name}: {rep}")


def test_large_logit_scale():
    """W_U with std 0.3: logits of tens of nats, sharply peaked rows, entropy near zero for some."""
    say("large logit scale")
    cfg = WL.LensConfig("peaked", L=2, T=150, d=256, V=3000, k=8)
    w = WL.make_workload(cfg, DEV, seed=5)
    w.W_U = (w.W_U.float() * 15.0).to(torch.bfloat16)
    got = run_project(w)
    ref = oracle_for(w, np.arange(cfg.N))
    P.compare(got, ref, cfg.k, label="peaked")
    assert ref["entropy"].min() < 1.0


# ------------------------------------------------------------------------------------------
# degenerate inputs
# ------------------------------------------------------------------------------------------
def test_empty_input_is_a_noop():
    say("N = 0")
    w = WL.make_workload(WL.LensConfig("e", L=1, T=4, d=64, V=300, k=3), DEV)
    empty = w.hidden.reshape(-1, 64)[:0]
    ids, p, logp, ent = project(empty, w.gamma, w.W_U, 1e-5, 3, w.target_ids[:0])
    torch.cuda.synchronize()
    assert ids.shape == (0, 3) and ent.shape == (0,)


def test_zero_rows_are_uniform_and_bad_targets_give_nan():
    say("zero rows, out-of-range targets")
    cfg = WL.LensConfig("z", L=1, T=70, d=128, V=700, k=6)
    w = WL.make_workload(cfg, DEV, seed=2)
    w.hidden[0, 5] = 0
    w.hidden[0, 69] = 0
    w.target_ids[3] = -1
    w.target_ids[4] = cfg.V
    w.target_ids[5] = cfg.V - 1
    got = run_project(w)
    for r in (5, 69):
        assert list(got["topk_ids"][r]) == list(range(6))          # all logits equal: ascending id
        np.testing.assert_allclose(got["topk_p"][r], 1.0 / cfg.V, rtol=1e-5)
        assert abs(got["entropy"][r] - math.log(cfg.V)) < 1e-5
    assert abs(got["target_logp"][5] + math.log(cfg.V)) < 1e-5
    assert np.isnan(got["target_logp"][3]) and np.isnan(got["target_logp"][4])
    ref = oracle_for(w, np.arange(cfg.N))
    P.compare(got, ref, cfg.k, label="zero-rows")


def test_a_non_finite_row_leaves_the_other_rows_alone():
    """Rows are independent: a row holding NaN or infinity must change no other row's result, on either side of a
    row-block boundary (the rows share workgroups, accumulator tiles and the merge kernel's blocks)."""
    say("non-finite rows")
    cfg = WL.LensConfig("nf", L=2, T=200, d=256, V=3000, k=8, n_outliers=2, outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=9)
    clean = run_project(w)
    h = w.hidden.reshape(-1, cfg.d)
    bad = {3: float("nan"), 255: float("inf"), 256: float("-inf"), 399: float("nan")}
    for r, val in bad.items():
        h[r, 17] = val
    got = run_project(w)
    keep = np.array([r for r in range(cfg.N) if r not in bad])
    for key in ("topk_ids", "topk_p", "target_logp", "entropy"):
        np.testing.assert_array_equal(got[key][keep], clean[key][keep], err_msg=key)
    for r in bad:                                   # the row itself: no claim beyond "not a number"
        assert np.isnan(got["entropy"][r])


def test_exact_ties_break_by_ascending_id():
    """Duplicate vocabulary rows give exactly equal logits: the smaller id must come first."""
    say("exact ties")
    cfg = WL.LensConfig("ties", L=1, T=64, d=128, V=600, k=8)
    w = WL.make_workload(cfg, DEV, seed=4)
    w.W_U[300:600] = w.W_U[0:300]                                   # id v and v+300 tie exactly (different tiles)
    w.W_U[1] = w.W_U[0]                                             # and two neighbours in one tile
    got = run_project(w)
    ref = oracle_for(w, np.arange(cfg.N))
    P.compare(got, ref, cfg.k, label="ties")
    ids = got["topk_ids"].astype(np.int64)
    diff = ids[:, 1:] - ids[:, :-1]
    # a duplicated row's two ids sit next to each other (equal logits), smaller id first
    assert np.sum(diff == 300) >= cfg.N and np.sum(diff == -300) == 0
    for r in range(cfg.N):
        row = list(ids[r])
        for v in row:
            if 1 < v < 300:
                if v + 300 in row:
                    assert row.index(v + 300) == row.index(v) + 1
                else:
                    assert row.index(v) == cfg.k - 1
        if 0 in row and 1 in row:
            assert row.index(0) < row.index(1)


def test_no_target_and_prenormalised_rows():
    say("target_ids = NULL; gamma = NULL")
    cfg = WL.LensConfig("nt", L=2, T=80, d=256, V=900, k=5)
    w = WL.make_workload(cfg, DEV, seed=6)
    got = run_project(w, target=False)
    ref = oracle_for(w, np.arange(cfg.N))
    P.compare(got, ref, cfg.k, has_target=False, label="no-target")
    # gamma = NULL: rows are used as they are
    res = project(w.hidden, None, w.W_U, cfg.eps, cfg.k, w.target_ids)
    torch.cuda.synchronize()
    got = P.to_numpy(res)
    ref = oracle_for(w, np.arange(cfg.N), gamma=None)
    P.compare(got, ref, cfg.k, label="gamma-null")


def test_paper_output_format_bias_and_topk_softmax():
    """ll_project_ex: the b of Eq. (1), and probabilities over the k selected logits only (paper Sec. 3.3)."""
    say("ll_project_ex: bias + top-k-only softmax")
    cfg = WL.LensConfig("ex", L=2, T=150, d=320, V=1300, k=3)       # k = 3 as in the paper's heatmap figure
    w = WL.make_workload(cfg, DEV, seed=8)
    g = torch.Generator(device=DEV).manual_seed(3)
    bias = torch.randn((cfg.V,), generator=g, device=DEV) * 0.5
    rows = np.arange(cfg.N)
    hb, gb, wb = WL.bf16_bits(w.hidden.reshape(-1, cfg.d)), WL.bf16_bits(w.gamma), WL.bf16_bits(w.W_U)
    t = w.target_ids.cpu().numpy()
    ref = P.oracle_rows(hb, gb, wb, cfg.eps, cfg.k, t, bias=bias.cpu().numpy())
    # bias only: full-softmax probabilities
    res = project(w.hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, bias=bias)
    torch.cuda.synchronize()
    P.compare(P.to_numpy(res), ref, cfg.k, label="bias")
    # bias + the paper's probabilities
    res = project(w.hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, bias=bias, topk_softmax=True)
    torch.cuda.synchronize()
    got = P.to_numpy(res)
    want_p = O.topk_renormalised(ref["topk_p"])
    assert np.max(np.abs(got["topk_p"] - want_p)) <= P.TOL_P
    np.testing.assert_allclose(got["topk_p"].sum(1), 1.0, atol=1e-5)
    P.validate_ids(got["topk_ids"], ref, "bias + top-k softmax")              # equal, or a near-tie of the oracle's logits
    big = want_p > P.P_FLOOR
    assert np.max(np.abs(np.log(got["topk_p"][big].astype(np.float64)) - np.log(want_p[big]))) <= P.TOL_LOG_P
    assert np.max(np.abs(got["entropy"] - ref["entropy"])) <= P.TOL_ENT      # still full-vocabulary
    assert np.max(np.abs(got["target_logp"] - ref["target_logp"])) <= P.TOL_LOGP
    # no bias, flag only, equals renormalising the plain result
    a = project(w.hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids)
    b = project(w.hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, topk_softmax=True)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0])
    assert torch.allclose(b[1], a[1] / a[1].sum(1, keepdim=True), atol=1e-6)


def test_caller_workspace_and_stream():
    say("caller-provided workspace on a side stream, twice")
    cfg = WL.LensConfig("ws", L=1, T=300, d=192, V=1500, k=4)
    w = WL.make_workload(cfg, DEV, seed=7)
    need = LL.ll_workspace_bytes(cfg.N, cfg.d, cfg.V, cfg.k)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)                                                  # stale contents must not matter
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        a = project(w.hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, workspace=ws, stream=s)
        b = project(w.hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, workspace=ws, stream=s)
    s.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    ref = oracle_for(w, np.arange(cfg.N))
    P.compare(P.to_numpy(a), ref, cfg.k, label="workspace")
    with pytest.raises(LL.LLError) as e:
        project(w.hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, workspace=ws[:need - 256])
    assert e.value.code == LL.LL_EWORKSPACE


def test_timed_variant_matches(gemm_path):
    if gemm_path != 2:
        pytest.skip("ll_project_timed has no kernel-choice argument")
    say("ll_project_timed")
    w = WL.make_workload("tiny", DEV)
    a = project(w.hidden, w.gamma, w.W_U, 1e-5, 5, w.target_ids)
    b = project(w.hidden, w.gamma, w.W_U, 1e-5, 5, w.target_ids, timed=True)
    torch.cuda.synchronize()
    for x, y in zip(a, b[:4]):
        assert torch.equal(x, y)
    assert len(b[4]) == 3 and all(t >= 0 for t in b[4]) and b[4][1] > 0


# ------------------------------------------------------------------------------------------
# the paper-shaped configs at full size, in the launch configuration the benchmark times:
# sampled rows against the oracle, every row against the invariants
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["qwen3-4b", "llama31-8b", "qwen3-32b", "llama31-70b"])
def test_full_size_config_sampled_rows(name, gemm_path):
    # The default kernel (the configuration the benchmark times) runs all four; the register-staged kernel, with the
    # norm applied inside the A-tile load, runs the first of them at full size on a smaller row sample.
    if gemm_path != 2 and name != "qwen3-4b":
        pytest.skip("the register-staged kernel runs one full-size config (qwen3-4b); the others are the default kernel's")
    cfg = WL.CONFIGS[name]
    say(f"full size {name}: N={cfg.N} d={cfg.d} V={cfg.V} k={cfg.k}, kernel path {gemm_path}")
    w = WL.make_workload(cfg, DEV)
    got = run_project(w)
    P.check_invariants(got, cfg.V, cfg.k, label=name)
    rows = WL.sample_rows(cfg, 256 if gemm_path == 2 else 64)
    ref = oracle_for(w, rows)
    rep = P.compare(P.take(got, rows), ref, cfg.k, label=name)
    say(f"{name}: {P.R1_STATEMENT}")
    say(f"{name}: against the gate oracle: {rep}")
    if gemm_path == 2:
        sub = rows[:: max(1, len(rows) // 64)]
        hb = WL.bf16_bits(w.hidden.reshape(-1, cfg.d)[torch.as_tensor(sub, device=DEV)])
        unr = P.oracle_rows(hb, WL.bf16_bits(w.gamma), WL.bf16_bits(w.W_U), cfg.eps, cfg.k,
                            w.target_ids.cpu().numpy()[sub], round_a=False)
        say(f"{name}: deviation from the un-rounded oracle on {len(sub)} rows (reported, not gated): "
            f"{P.deviation_from_unrounded(P.take(got, sub), unr)}")
    # the Gaussian unembedding predicts the mean entropy: log V - var(z)/2 (a sanity band, not the gate)
    a = O.rmsnorm(WL.bf16_bits(w.hidden.reshape(-1, cfg.d)[torch.as_tensor(rows, device=DEV)]),
                  WL.bf16_bits(w.gamma), cfg.eps)
    pred = math.log(cfg.V) - 0.5 * 0.02 ** 2 * np.sum(a * a, axis=1)
    assert abs(float(np.mean(got["entropy"][rows])) - float(np.mean(pred))) < 0.05
    del w
    torch.cuda.empty_cache()


def test_full_size_paper_output_format(gemm_path):
    """ll_project_ex at the size the headline metric is quoted on: Eq. (1) with its bias b, probabilities over the
    k = 3 selected logits only (Sec. 3.3, the format of the paper's heatmaps), sampled rows against the oracle."""
    if gemm_path != 2:
        pytest.skip("the default kernel is the one a bias selects; the other kernel's bias path is covered at small sizes")
    cfg = WL.CONFIGS["llama31-70b"]
    k = 3
    say(f"full size ll_project_ex llama31-70b: bias + top-k-only softmax, k={k}")
    w = WL.make_workload(cfg, DEV)
    g = torch.Generator(device=DEV).manual_seed(17)
    bias = torch.randn((cfg.V,), generator=g, device=DEV) * 0.5
    res = project(w.hidden, w.gamma, w.W_U, cfg.eps, k, w.target_ids, bias=bias, topk_softmax=True)
    torch.cuda.synchronize()
    got = P.to_numpy(res)
    rows = WL.sample_rows(cfg, 128)
    hb = WL.bf16_bits(w.hidden.reshape(-1, cfg.d)[torch.as_tensor(rows, device=DEV)])
    ref = P.oracle_rows(hb, WL.bf16_bits(w.gamma), WL.bf16_bits(w.W_U), cfg.eps, k, w.target_ids.cpu().numpy()[rows],
                        bias=bias.cpu().numpy())
    sub = P.take(got, rows)
    P.validate_ids(sub["topk_ids"], ref, "70B ll_project_ex")
    want_p = O.topk_renormalised(ref["topk_p"])
    assert np.max(np.abs(sub["topk_p"] - want_p)) <= P.TOL_P
    assert np.max(np.abs(np.log(sub["topk_p"].astype(np.float64)) - np.log(want_p))) <= P.TOL_LOG_P
    np.testing.assert_allclose(got["topk_p"].sum(1), 1.0, atol=1e-5)            # every row: a distribution over the k
    assert np.max(np.abs(sub["entropy"] - ref["entropy"])) <= P.TOL_ENT         # still full-vocabulary
    assert np.max(np.abs(sub["target_logp"] - ref["target_logp"])) <= P.TOL_LOGP
    # the bias matters at this size: without it the sampled rows' entropies differ by far more than the tolerance
    plain = project(w.hidden, w.gamma, w.W_U, cfg.eps, k, w.target_ids)
    torch.cuda.synchronize()
    assert np.max(np.abs(plain[3].cpu().numpy()[rows] - ref["entropy"])) > 10 * P.TOL_ENT
    del w
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------------
# the projection allocates nothing and never synchronises: it can be captured in a HIP graph
# ------------------------------------------------------------------------------------------
def test_projection_replays_from_a_hip_graph(gemm_path):
    if gemm_path != 2:
        pytest.skip("one kernel path is enough for this property")
    say("graph capture")
    cfg = WL.LensConfig("graph", L=2, T=300, d=256, V=5000, k=10, n_outliers=4, outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=4)
    N = cfg.N
    ws = torch.empty(LL.ll_workspace_bytes(N, cfg.d, cfg.V, cfg.k), dtype=torch.uint8, device=DEV)
    out = (torch.zeros((N, cfg.k), dtype=torch.int32, device=DEV), torch.zeros((N, cfg.k), dtype=torch.float32, device=DEV),
           torch.zeros((N,), dtype=torch.float32, device=DEV), torch.zeros((N,), dtype=torch.float32, device=DEV))
    hidden = w.hidden.clone()
    eager = [t.clone() for t in project(hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids)]
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        project(hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, workspace=ws, out=out, stream=s)   # warm-up
        s.synchronize()
        with torch.cuda.graph(g, stream=s):
            project(hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids, workspace=ws, out=out, stream=s)
    for rep in range(3):
        for t in out:
            t.zero_()
        ws.zero_()                                   # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip(out, eager):
            assert torch.equal(got, want), f"replay {rep} differs from the eager result"
    # new input in the captured buffer, same graph
    hidden.copy_(torch.flip(w.hidden, dims=(1,)))
    want = [t.clone() for t in project(hidden, w.gamma, w.W_U, cfg.eps, cfg.k, w.target_ids)]
    g.replay()
    torch.cuda.synchronize()
    for got, w_ in zip(out, want):
        assert torch.equal(got, w_)
