"""ll_project_static (the entry point that allocates nothing: its workspace is a device array inside the
library) against ll_project, through the C ABI, on two calls in a row, the second with a smaller input."""
import sys

import pytest
import torch

from paper_2604_06483_amd import binding as LL
from paper_2604_06483_amd import workloads as WL

from tests.conftest import say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"



def both(cfg, seed):
    w = WL.make_workload(cfg, DEV, seed=seed)
    N, k = cfg.N, cfg.k
    out = (torch.full((N, k), -7, dtype=torch.int32, device=DEV), torch.full((N, k), -7.0, dtype=torch.float32, device=DEV),
           torch.full((N,), -7.0, dtype=torch.float32, device=DEV), torch.full((N,), -7.0, dtype=torch.float32, device=DEV))
    got = LL.ll_project_static(w.hidden, w.gamma, w.W_U, cfg.eps, k, w.target_ids, out=out)
    want = LL.ll_project(w.hidden, w.gamma, w.W_U, cfg.eps, k, w.target_ids)
    torch.cuda.synchronize()
    return got, want


def test_same_passes_bit_identical_two_calls_second_smaller():
    """Shapes whose 8192-row plan fits the static buffer run the very same launches as ll_project: equal bits.
    The second call is smaller in every dimension and finds the first one's partials in the buffer."""
    first = WL.LensConfig("static-a", L=3, T=300, d=320, V=5000, k=12, n_outliers=2, outlier_scale=20.0)
    second = WL.LensConfig("static-b", L=1, T=130, d=128, V=1300, k=5)
    for cfg, seed in ((first, 11), (second, 12)):
        say(f"ll_project_static {cfg.name}: N={cfg.N} d={cfg.d} V={cfg.V} k={cfg.k}")
        assert LL.ll_project_static_pass_rows(cfg.N, cfg.d, cfg.V, cfg.k) == 8192
        got, want = both(cfg, seed)
        for name, g, w_ in zip(("ids", "p", "logp", "entropy"), got, want):
            assert torch.equal(g, w_), f"{cfg.name}: {name} differs from ll_project"


def test_smaller_passes_same_logits_two_calls_second_smaller():
    """d = 8192, k = 20: the 8192-row plan does not fit, the rows go in smaller passes with more vocabulary splits.
    Every logit is accumulated in the same order, so ids are identical; the softmax sums are merged from other
    partials, so the floating-point results agree to fp32 rounding of those sums."""
    first = WL.LensConfig("static-c", L=7, T=500, d=8192, V=3000, k=20, n_outliers=4, outlier_scale=20.0)
    second = WL.LensConfig("static-d", L=4, T=865, d=8192, V=2500, k=20, n_outliers=4, outlier_scale=20.0)
    for cfg, seed in ((first, 13), (second, 14)):
        rows = LL.ll_project_static_pass_rows(cfg.N, cfg.d, cfg.V, cfg.k)
        say(f"ll_project_static {cfg.name}: N={cfg.N} d={cfg.d} V={cfg.V} k={cfg.k}, passes of {rows} rows")
        assert 0 < rows < 8192
        got, want = both(cfg, seed)
        assert torch.equal(got[0], want[0]), f"{cfg.name}: ids differ from ll_project"
        assert torch.allclose(got[1], want[1], rtol=2e-5, atol=1e-9), f"{cfg.name}: probabilities"
        assert torch.allclose(got[2], want[2], rtol=0, atol=2e-5), f"{cfg.name}: target log-prob"
        assert torch.allclose(got[3], want[3], rtol=0, atol=2e-5), f"{cfg.name}: entropy"
        assert cfg.N > rows                                                                    # more than one pass
    # one decoding step's rows (the newest token of every layer) at the same hidden size: a single ordinary pass
    step = WL.LensConfig("static-step", L=81, T=1, d=8192, V=2500, k=20, n_outliers=4, outlier_scale=20.0)
    say(f"ll_project_static {step.name}: N={step.N}")
    got, want = both(step, 15)
    for g, w_ in zip(got, want):
        assert torch.equal(g, w_)


def test_oversized_shape_is_refused():
    say("ll_project_static: 300 rows of d = 2^18 do not fit")
    d = 1 << 18
    h = torch.empty((300, d), dtype=torch.bfloat16, device=DEV)
    w = torch.empty((64, d), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(LL.LLError) as e:
        LL.ll_project_static(h, None, w, 1e-5, 3)
    assert e.value.code == LL.LL_ESCRATCH


def test_replays_from_a_hip_graph_between_other_calls():
    """The callers this entry point is for: one decoding step's rows, captured once and replayed, with other calls
    on the same static buffer (a different shape, several passes) between the replays.  Every replay gives the
    eager call's bits."""
    step = WL.LensConfig("static-graph", L=81, T=1, d=1024, V=70000, k=20, n_outliers=4, outlier_scale=20.0)
    other = WL.LensConfig("static-between", L=2, T=300, d=8192, V=1500, k=20)
    say(f"ll_project_static under graph capture: N={step.N} d={step.d} V={step.V} k={step.k}")
    w = WL.make_workload(step, DEV, seed=16)
    wo = WL.make_workload(other, DEV, seed=17)
    N, k = step.N, step.k
    hidden = w.hidden.clone()
    out = (torch.zeros((N, k), dtype=torch.int32, device=DEV), torch.zeros((N, k), dtype=torch.float32, device=DEV),
           torch.zeros((N,), dtype=torch.float32, device=DEV), torch.zeros((N,), dtype=torch.float32, device=DEV))
    eager = [t.clone() for t in LL.ll_project(hidden, w.gamma, w.W_U, step.eps, k, w.target_ids)]
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        LL.ll_project_static(hidden, w.gamma, w.W_U, step.eps, k, w.target_ids, out=out, stream=s)   # first use: set-up
        s.synchronize()
        with torch.cuda.graph(g, stream=s):
            LL.ll_project_static(hidden, w.gamma, w.W_U, step.eps, k, w.target_ids, out=out, stream=s)
    for rep in range(3):
        for t in out:
            t.zero_()
        LL.ll_project_static(wo.hidden, wo.gamma, wo.W_U, other.eps, other.k, wo.target_ids)   # scribbles on the buffer
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("ids", "p", "logp", "entropy"), out, eager):
            assert torch.equal(got, want), f"replay {rep}: {name} differs from the eager ll_project"
    hidden.copy_(torch.flip(w.hidden, dims=(0,)))                   # new rows in the captured buffer, same graph
    want = [t.clone() for t in LL.ll_project(hidden, w.gamma, w.W_U, step.eps, k, w.target_ids)]
    g.replay()
    torch.cuda.synchronize()
    for got, w_ in zip(out, want):
        assert torch.equal(got, w_)
