"""Host-side checks of the synthetic workload generator and of the size arithmetic the
benchmark reports (the paper's Sec. 3.2 memory example is the fixture)."""
import os

import numpy as np
import torch

from paper_2604_06483_amd import workloads as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "memory_example.txt")


def _golden():
    vals = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        vals[k] = float(v)
    return vals


def test_memory_example_of_the_paper():
    """Sec. 3.2: T=1500, d=8192, 80 layers -> about 9.8e8 elements, about 1.97 GB in bf16."""
    g = _golden()
    elements = g["T"] * g["d"] * g["layers"]
    assert abs(elements - g["elements_approx"]) / elements < 0.01
    gb = elements * g["bytes_per_element"] / 1e9
    assert abs(gb - g["gigabytes_per_activation_type_approx"]) < 0.005
    assert abs(3 * gb - g["gigabytes_three_types_approx"]) < 0.01
    # the 70B-shaped config is that example plus the embedding output
    cfg = WL.CONFIGS["llama31-70b"]
    assert (cfg.T, cfg.d, cfg.L - 1) == (g["T"], g["d"], g["layers"])
    assert cfg.hidden_bytes == (elements + cfg.T * cfg.d) * 2


def test_config_table():
    n = {k: c.N for k, c in WL.CONFIGS.items()}
    assert n == {"tiny": 64, "qwen3-4b": 55500, "llama31-8b": 49500, "qwen3-32b": 97500, "llama31-70b": 121500}
    assert abs(WL.CONFIGS["llama31-70b"].flop - 2.553e14) / 2.553e14 < 1e-3
    assert abs(WL.CONFIGS["llama31-70b"].w_bytes - 2.101e9) / 2.101e9 < 1e-3


def test_tiny_workload_is_seeded_and_shaped():
    a = WL.make_workload("tiny", "cpu", seed=0)
    b = WL.make_workload("tiny", "cpu", seed=0)
    c = WL.make_workload("tiny", "cpu", seed=1)
    assert a.hidden.shape == (4, 16, 256) and a.hidden.dtype == torch.bfloat16
    assert a.W_U.shape == (4096, 256) and a.gamma.shape == (256,)
    assert a.target_ids.shape == (64,) and a.target_ids.dtype == torch.int32
    assert torch.equal(a.hidden, b.hidden) and torch.equal(a.W_U, b.W_U)
    assert not torch.equal(a.hidden, c.hidden)
    assert int(a.target_ids.min()) >= 0 and int(a.target_ids.max()) < 4096
    # per-layer scale 1 + l and W_U std 0.02
    std = a.hidden.float().std(dim=(1, 2))
    assert torch.allclose(std, torch.tensor([1.0, 2.0, 3.0, 4.0]), rtol=0.05)
    assert abs(float(a.W_U.float().std()) - 0.02) < 1e-3
    assert abs(float(a.gamma.float().mean()) - 1.0) < 0.03


def test_outlier_channels():
    cfg = WL.LensConfig("mini", L=3, T=40, d=128, V=64, k=4, n_outliers=4, outlier_scale=20.0)
    w = WL.make_workload(cfg, "cpu")
    assert len(set(w.outlier_idx.tolist())) == 4
    std = w.hidden.float().std(dim=(0, 1))
    mask = torch.zeros(128, dtype=torch.bool)
    mask[w.outlier_idx] = True
    assert std[mask].min() > 5 * std[~mask].max()


def test_bits_roundtrip_and_row_sample():
    t = torch.randn(5, 7).to(torch.bfloat16)
    bits = WL.bf16_bits(t)
    assert bits.dtype == np.uint16 and torch.equal(WL.bits_to_bf16(bits), t)
    cfg = WL.CONFIGS["llama31-70b"]
    rows = WL.sample_rows(cfg, 512)
    assert len(rows) == 512 and len(set(rows.tolist())) == 512
    assert rows[0] == 0 and rows[-1] == cfg.N - 1
    assert {8192 * i for i in range(15)} <= set(rows.tolist())
    assert {8192 * i - 1 for i in range(1, 15)} <= set(rows.tolist())
    assert set(rows // cfg.T) == set(range(cfg.L))
    assert np.array_equal(WL.sample_rows(cfg, 512), rows)
    assert np.array_equal(WL.sample_rows("tiny", 512), np.arange(64))


def test_steer_rows():
    cfg = WL.LensConfig("mini", L=4, T=8, d=256, V=64, k=4, n_outliers=2, outlier_scale=20.0)
    w = WL.make_workload(cfg, "cpu")
    base, target, l_star = WL.make_steer_rows(cfg, w.outlier_idx, "cpu")
    assert base.shape == (64, 256) and target.shape == (64, 256) and l_star == 2
    assert base.dtype == torch.bfloat16
    assert float((target.float().mean(0) - base.float().mean(0)).norm()) > 1.0


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N with N > 1 exits with a message that says so (no GPU needed for this)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "ONE GPU" in (res.stdout + res.stderr)
