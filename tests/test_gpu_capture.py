"""Capture store (paper Sec. 3.1 Stage 2/3) and the in-model injection with its safeguards (Sec. 3.4)
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



@pytest.mark.parametrize("L,C,T,d,steps", [
    (4, 3, 40, 512, (17, 1, 1, 1, 5, 1, 14)),      # a prefill, decoding steps, a chunk, up to capacity
    (1, 1, 9, 8, (1,) * 9),                        # smallest rows
    (7, 3, 33, 8192, (30, 1, 1, 1)),               # 16 KB rows, prefill-sized append
    (2, 2, 300, 328, (299, 1)),                    # d not a multiple of 64
])
def test_capture_append_builds_the_trajectories(L, C, T, d, steps):
    say(f"capture_append L={L} C={C} T={T} d={d} steps={steps}")
    assert sum(steps) == T
    g = torch.Generator(device=DEV).manual_seed(L * 100 + T)
    store = torch.full((L, C, T, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    slices, t0 = [], 0
    for n in steps:
        s = torch.randn((L * C, n, d), generator=g, device=DEV).to(torch.bfloat16)
        LL.ll_capture_append(store, s, t0)
        slices.append(WL.bf16_bits(s))
        t0 += n
    torch.cuda.synchronize()
    want = O.concat_trajectories(slices, L, C)
    assert np.array_equal(WL.bf16_bits(store), want)            # a copy: bit for bit
    # an append in the middle touches only its own tokens
    before = WL.bf16_bits(store).copy()
    s = torch.randn((L * C, 2, d), generator=g, device=DEV).to(torch.bfloat16)
    LL.ll_capture_append(store, s, 3)
    torch.cuda.synchronize()
    after = WL.bf16_bits(store)
    before[:, :, 3:5, :] = WL.bf16_bits(s).reshape(L, C, 2, d)
    assert np.array_equal(after, before)
    with pytest.raises(LL.LLError):
        LL.ll_capture_append(store, s, T - 1)                    # would run past the capacity


def test_captured_store_is_what_the_projection_reads():
    """Three activation types captured step by step, then decoded in one call over the whole store."""
    say("capture -> project")
    L, C, T, d, V, k = 3, 3, 50, 256, 3000, 5
    cfg = WL.LensConfig("cap", L=L * C, T=T, d=d, V=V, k=k, n_outliers=4, outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV, seed=2)
    traj = w.hidden.reshape(L * C, T, d)
    store = torch.zeros((L, C, T, d), dtype=torch.bfloat16, device=DEV)
    LL.ll_capture_append(store, traj[:, :20].contiguous(), 0)
    for t in range(20, T):
        LL.ll_capture_append(store, traj[:, t:t + 1].contiguous(), t)
    got = LL.ll_project(store.reshape(-1, d), w.gamma, w.W_U, cfg.eps, k, w.target_ids)
    ref = LL.ll_project(w.hidden, w.gamma, w.W_U, cfg.eps, k, w.target_ids)
    torch.cuda.synchronize()
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
    rows = np.arange(0, L * C * T, 7)
    want = P.oracle_rows(WL.bf16_bits(store.reshape(-1, d))[rows], WL.bf16_bits(w.gamma), WL.bf16_bits(w.W_U), cfg.eps, k,
                         w.target_ids.cpu().numpy()[rows])
    P.compare(P.take(P.to_numpy(got), rows), want, k, label="captured store")


def test_three_activation_types_at_the_papers_size():
    """The capture store of the paper's memory example (Sec. 3.2: T = 1500, d = 8192, 80 layers, attention + MLP +
    block outputs, about 5.9 GB) with the embedding output on top: 81 x 3 trajectories = 364 500 lens rows.  Filled
    the way generation fills it (a prefill-sized append, then single-token decoding steps, then a multi-token
    chunk), it must equal the concatenated slices bit for bit, and the projection reads it as it stands: sampled
    rows against the oracle, every row against the invariants."""
    base = WL.CONFIGS["llama31-70b"]
    L, C, T, d, V, k = base.L, 3, base.T, base.d, base.V, base.k
    say(f"capture -> project at full size: L={L} C={C} T={T} d={d} ({L * C * T} rows, {L * C * T * d * 2 / 1e9:.2f} GB)")
    cfg = WL.LensConfig("capture-3types", L=L * C, T=T, d=d, V=V, k=k, n_outliers=4, outlier_scale=20.0)
    w = WL.make_workload(cfg, DEV)                                # trajectory (l, c) = "layer" l * C + c of this workload
    store = torch.full((L, C, T, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    t = 0
    for n in (1200,) + (1,) * 40 + (260,):                        # prefill, 40 decoding steps, a trailing chunk
        LL.ll_capture_append(store, w.hidden[:, t:t + n].contiguous(), t)
        t += n
    assert t == T
    torch.cuda.synchronize()
    assert torch.equal(store.reshape(L * C, T, d).view(torch.int16), w.hidden.view(torch.int16))     # a copy: bit for bit
    del w.hidden
    res = LL.ll_project(store, w.gamma, w.W_U, cfg.eps, k, w.target_ids)
    torch.cuda.synchronize()
    got = P.to_numpy(res)
    P.check_invariants(got, V, k, label="capture-3types")
    rows = WL.sample_rows(cfg, 96)
    hb = WL.bf16_bits(store.reshape(-1, d)[torch.as_tensor(rows, device=DEV)])
    ref = P.oracle_rows(hb, WL.bf16_bits(w.gamma), WL.bf16_bits(w.W_U), cfg.eps, k, w.target_ids.cpu().numpy()[rows])
    rep = P.compare(P.take(got, rows), ref, k, label="capture-3types")
    say(f"capture-3types: {rep}")
    del store, w
    torch.cuda.empty_cache()


@pytest.mark.parametrize("N,d", [(300, 4096), (7, 328), (130, 8192), (33, 64), (20, 9000)])
def test_steer_inject_raw(N, d):
    say(f"steer_inject_raw N={N} d={d}")
    g = torch.Generator(device=DEV).manual_seed(N + d)
    h = (3 * torch.randn((N, d), generator=g, device=DEV)).to(torch.bfloat16)
    h[0] = 0                                                     # a zero row: the cap is zero
    v = torch.randn((d,), generator=g, device=DEV)
    v = v / v.norm()
    hb = WL.bf16_bits(h)
    for alpha, scale, clip in ((2.5, 1.0, 0.0), (-4.0, 0.5, 0.0), (50.0, 1.0, 0.1), (-50.0, 2.0, 0.05), (0.3, 1.0, 0.5)):
        out = LL.ll_steer_inject_raw(h, v, alpha, scale, clip)
        torch.cuda.synchronize()
        got = O.bf16_bits_to_f64(WL.bf16_bits(out))
        want = O.bf16_bits_to_f64(O.steer_inject_raw(hb, v.cpu().numpy(), alpha, scale, clip))
        # fp32 norm and fma before the one bf16 rounding: at most one bf16 step where the sum sits on a rounding boundary
        hf = O.bf16_bits_to_f64(hb)
        bound = np.abs(want) * 2.0 ** -7 + (np.abs(hf) + abs(alpha * scale) * np.abs(v.cpu().numpy())[None, :]) * 2.0 ** -20
        assert np.all(np.abs(got - want) <= bound), f"alpha={alpha} clip={clip}"
        assert (got != want).mean() < 5e-3
        if clip > 0:
            assert np.array_equal(got[0], np.zeros(d))           # nothing may be added to a zero row
    h2 = h.clone()
    LL.ll_steer_inject_raw(h2, v, 2.5, 1.0, 0.2, out=h2)          # in place
    torch.cuda.synchronize()
    assert torch.equal(h2, LL.ll_steer_inject_raw(h, v, 2.5, 1.0, 0.2))
