"""Seeded synthetic inputs for the logit-lens projection and steering calls.

This module draws random tensors and picks row indices; it holds none of the
method's arithmetic (no normalisation, projection, softmax or steering maths)
so that both the HIP library's callers and the CPU checker can take their
inputs from it without sharing anything else.

The shapes stand in for the paper's runs (Sec. 4: LLaMA-3.1 8B/70B and Qwen3
4B/32B, all layers traced, 1,500-token sequences; Sec. 3.2 memory example:
T=1500, d=8192, 80 layers).  The model checkpoints, the prompt suite and the
steering datasets are not reproduced: hidden states are Gaussian with a
per-layer scale and a few fixed outlier channels, the unembedding is Gaussian.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch


@dataclass(frozen=True)
class LensConfig:
    name: str
    L: int                  # captured states (embedding output + layers)
    T: int                  # tokens per trajectory
    d: int                  # hidden size
    V: int                  # vocabulary size
    k: int                  # top-k
    sigma: str = "ramp"     # "ramp": 1 + 4 l / L ; "linear": 1 + l
    n_outliers: int = 0     # channels scaled by outlier_scale in every row
    outlier_scale: float = 1.0
    eps: float = 1e-5
    chunk_rows: int = 8192  # rows per projection pass

    @property
    def N(self) -> int:
        return self.L * self.T

    @property
    def flop(self) -> float:
        return 2.0 * self.N * self.d * self.V

    @property
    def hidden_bytes(self) -> int:
        return self.N * self.d * 2

    @property
    def w_bytes(self) -> int:
        return self.V * self.d * 2


CONFIGS = {
    "tiny": LensConfig("tiny", L=4, T=16, d=256, V=4096, k=5, sigma="linear"),
    "qwen3-4b": LensConfig("qwen3-4b", L=37, T=1500, d=2560, V=151936, k=10,
                           n_outliers=4, outlier_scale=20.0),
    "llama31-8b": LensConfig("llama31-8b", L=33, T=1500, d=4096, V=128256, k=10,
                             n_outliers=4, outlier_scale=20.0),
    "qwen3-32b": LensConfig("qwen3-32b", L=65, T=1500, d=5120, V=151936, k=20,
                            n_outliers=6, outlier_scale=30.0),
    "llama31-70b": LensConfig("llama31-70b", L=81, T=1500, d=8192, V=128256, k=20,
                              n_outliers=4, outlier_scale=20.0),
}

_STREAMS = ("hidden", "outlier_idx", "gamma", "W_U", "target_ids",
            "steer_base", "steer_target", "steer_offset", "row_sample")


def _gen(seed: int, stream: str, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000 + _STREAMS.index(stream))
    return g


def layer_sigma(cfg: LensConfig) -> torch.Tensor:
    l = torch.arange(cfg.L, dtype=torch.float32)
    return 1.0 + l if cfg.sigma == "linear" else 1.0 + 4.0 * l / cfg.L


@dataclass
class LensWorkload:
    cfg: LensConfig
    hidden: torch.Tensor        # [L, T, d] bf16
    gamma: torch.Tensor         # [d] bf16
    W_U: torch.Tensor           # [V, d] bf16
    target_ids: torch.Tensor    # [N] int32
    outlier_idx: torch.Tensor   # [n_outliers] int64 (CPU)
    extra: dict = field(default_factory=dict)


def _randn_bf16(shape, scale, gen, device, rows_per_block=4096):
    """bf16(scale * N(0,1)) drawn in fp32 blocks so the fp32 temporary stays small."""
    n0 = shape[0]
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    for r0 in range(0, n0, rows_per_block):
        r1 = min(n0, r0 + rows_per_block)
        blk = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen,
                          device=device, dtype=torch.float32)
        out[r0:r1] = (blk * scale).to(torch.bfloat16)
    return out


def make_workload(cfg, device="cpu", seed: int = 0) -> LensWorkload:
    """Draw hidden / gamma / W_U / target_ids for a config (name or LensConfig)."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    device = torch.device(device)
    sig = layer_sigma(cfg).to(device)

    g = _gen(seed, "hidden", device)
    hidden = torch.empty((cfg.L, cfg.T, cfg.d), dtype=torch.bfloat16, device=device)
    g_out = _gen(seed, "outlier_idx", "cpu")
    outlier_idx = torch.randperm(cfg.d, generator=g_out)[:cfg.n_outliers]
    for l in range(cfg.L):
        blk = torch.randn((cfg.T, cfg.d), generator=g, device=device, dtype=torch.float32)
        blk = blk * sig[l]
        if cfg.n_outliers:
            blk[:, outlier_idx.to(device)] *= cfg.outlier_scale
        hidden[l] = blk.to(torch.bfloat16)

    g = _gen(seed, "gamma", device)
    gamma = (1.0 + 0.1 * torch.randn((cfg.d,), generator=g, device=device,
                                     dtype=torch.float32)).to(torch.bfloat16)
    W_U = _randn_bf16((cfg.V, cfg.d), 0.02, _gen(seed, "W_U", device), device)
    g = _gen(seed, "target_ids", device)
    target_ids = torch.randint(0, cfg.V, (cfg.N,), generator=g, device=device,
                               dtype=torch.int32)
    return LensWorkload(cfg, hidden, gamma, W_U, target_ids, outlier_idx)


def make_steer_rows(cfg, outlier_idx, device="cpu", seed: int = 0,
                    n_base: int = 64, n_target: int = 64):
    """Base / target rows at the label position of the middle layer.

    Both are fresh rows with the middle layer's scale and the config's outlier
    channels; the target rows carry a fixed offset (a random unit direction
    times twice that scale) so that the two means really differ.
    Returns (base [n_base, d] bf16, target [n_target, d] bf16, layer index).
    """
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    device = torch.device(device)
    l_star = cfg.L // 2
    s = float(layer_sigma(cfg)[l_star])

    def rows(n, stream):
        g = _gen(seed, stream, device)
        r = torch.randn((n, cfg.d), generator=g, device=device, dtype=torch.float32) * s
        if cfg.n_outliers:
            r[:, outlier_idx.to(device)] *= cfg.outlier_scale
        return r

    g = _gen(seed, "steer_offset", device)
    u = torch.randn((cfg.d,), generator=g, device=device, dtype=torch.float32)
    u = u / u.norm() * (2.0 * s)
    base = rows(n_base, "steer_base").to(torch.bfloat16)
    target = (rows(n_target, "steer_target") + u).to(torch.bfloat16)
    return base, target, l_star


def sample_rows(cfg, R: int = 512, seed: int = 0) -> np.ndarray:
    """Sorted row indices for sampled checks: every layer is represented, rows 0
    and N-1 and the first/last row of every projection chunk are forced in, the
    rest is uniform."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    N = cfg.N
    if R >= N:
        return np.arange(N, dtype=np.int64)
    rng = np.random.Generator(np.random.PCG64(int(seed) * 1000 + _STREAMS.index("row_sample")))
    forced = {0, N - 1}
    for c0 in range(0, N, cfg.chunk_rows):
        forced.add(c0)
        forced.add(min(N, c0 + cfg.chunk_rows) - 1)
    for l in range(cfg.L):
        forced.add(l * cfg.T + int(rng.integers(0, cfg.T)))
    forced = sorted(forced)[:R]
    chosen = set(forced)
    while len(chosen) < R:
        for r in rng.integers(0, N, size=R - len(chosen)):
            chosen.add(int(r))
    return np.array(sorted(chosen), dtype=np.int64)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """The bit patterns of a bf16 tensor as a uint16 NumPy array (a host copy)."""
    assert t.dtype == torch.bfloat16
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_bf16(bits: np.ndarray, device="cpu") -> torch.Tensor:
    """Inverse of `bf16_bits`."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16)
    return torch.from_numpy(b.copy()).view(torch.bfloat16).to(device)
