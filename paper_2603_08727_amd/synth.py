"""Seeded synthetic workloads (inputs only; none of the method's arithmetic).

Stands in for the prompts the paper runs (LongBench / lm-eval on LLaMA3 and
Qwen3 checkpoints, Sec. V-B), which need datasets and weights that are not
available: tensors have the shapes of those models' KV caches and a value
structure that exercises the method (a few high-norm 'sink' keys, two outlier
key channels, optional planted heavy hitters, per-layer or per-head softmax
temperature).  Both the CPU oracle's tests and the HIP path's tests/benchmark
take their inputs from here; this module imports neither of them.

All tensors are bf16.  Randomness: torch.Generator on the requested device,
seed = base_seed + 1000*layer + tensor_id.  CPU and GPU generators produce
different streams, so a comparison always draws once and copies.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefill: int           # T
    decode_steps: int
    budget_frac: float     # N = floor(frac * T)
    bits: int = 4
    window: int = 32
    alpha: float = 0.75
    gamma: float = 263.81
    tau: tuple = (7.774, 5.407, 5.528)
    n_sinks: int = 4
    sink_gain: float = 8.0
    outlier_gain: float = 10.0
    layer_temp: tuple | None = None       # (lo, hi): per-layer temperature ~ U[lo, hi]
    head_temps: tuple | None = None       # (sharp, flat): per (layer, q-head) 50/50
    heavy_frac: float = 0.0               # fraction of prompt positions with keys x heavy_gain
    heavy_gain: float = 4.0
    seed: int = 0

    @property
    def capacity(self) -> int:
        return int(math.floor(self.budget_frac * self.prefill))

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five benchmark configurations, in the benchmark definition's order.
C1 = Workload("c1_small", 1, 1, 8, 2, 64, 512, 64, 0.25, bits=4)
C2 = Workload("c2_llama3_8b_8k", 32, 1, 32, 8, 128, 8192, 256, 0.25, bits=4)
C3 = Workload("c3_qwen3_8b_32k_b4", 36, 4, 32, 8, 128, 32768, 128, 0.25, bits=4, layer_temp=(0.5, 2.0))
C4 = Workload("c4_llama3_8b_128k_2bit", 32, 1, 32, 8, 128, 131072, 64, 0.125, bits=2, heavy_frac=0.01)
C5 = Workload("c5_prefill_scorer_16k_b8", 32, 8, 32, 8, 128, 16384, 0, 0.25, head_temps=(0.3, 3.0))
CONFIGS = {w.name: w for w in (C1, C2, C3, C4, C5)}


def _gen(wl: Workload, layer: int, tensor_id: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(wl.seed + 1000 * layer + tensor_id)
    return g


def _randn(shape, gen, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def _outlier_channels(d: int):
    return (3, d // 2 + 3)


def layer_temperature(wl: Workload, layer: int) -> float:
    if wl.layer_temp is None:
        return 1.0
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed + 1000 * layer + 7)
    lo, hi = wl.layer_temp
    return float(lo + (hi - lo) * torch.rand((), generator=g).item())


def softmax_scale(wl: Workload, layer: int) -> float:
    return 1.0 / (math.sqrt(wl.head_dim) * layer_temperature(wl, layer))


def prefill_inputs(wl: Workload, layer: int, device="cpu", batch_slice=None):
    """K, V [B, Hkv, T, d], Q_win [B, Hq, W, d] of one layer, bf16.
    batch_slice=(b0, b1) restricts to sequences b0..b1-1 of the same draw only
    when the device is the CPU; on a GPU the whole batch is drawn and sliced."""
    B, T, d = wl.batch, wl.prefill, wl.head_dim
    k = _randn((B, wl.n_kv_heads, T, d), _gen(wl, layer, 1, device), device)
    v = _randn((B, wl.n_kv_heads, T, d), _gen(wl, layer, 2, device), device)
    qw = _randn((B, wl.n_q_heads, wl.window, d), _gen(wl, layer, 3, device), device)
    k[:, :, : wl.n_sinks, :] *= wl.sink_gain
    for c in _outlier_channels(d):
        k[:, :, :, c] *= wl.outlier_gain
    if wl.heavy_frac > 0:
        g = torch.Generator(device="cpu")
        g.manual_seed(wl.seed + 1000 * layer + 8)
        n_heavy = max(1, int(wl.heavy_frac * T))
        idx = torch.randperm(T, generator=g)[:n_heavy].to(device)
        k[:, :, idx, :] *= wl.heavy_gain
    if wl.head_temps is not None:
        g = torch.Generator(device="cpu")
        g.manual_seed(wl.seed + 1000 * layer + 9)
        sharp = torch.rand(wl.n_q_heads, generator=g) < 0.5
        temps = torch.where(sharp, torch.tensor(wl.head_temps[0]), torch.tensor(wl.head_temps[1]))
        qw /= temps.to(device).view(1, -1, 1, 1)
    k, v, qw = k.to(torch.bfloat16), v.to(torch.bfloat16), qw.to(torch.bfloat16)
    if batch_slice is not None:
        b0, b1 = batch_slice
        k, v, qw = k[b0:b1], v[b0:b1], qw[b0:b1]
    return k.contiguous(), v.contiguous(), qw.contiguous()


def decode_inputs(wl: Workload, layer: int, steps: int | None = None, device="cpu"):
    """q [S, B, Hq, d], k_new, v_new [S, B, Hkv, d] for S decode steps, bf16.
    New keys carry the outlier channels (not the sink gain)."""
    S = wl.decode_steps if steps is None else steps
    B, d = wl.batch, wl.head_dim
    q = _randn((S, B, wl.n_q_heads, d), _gen(wl, layer, 4, device), device)
    kn = _randn((S, B, wl.n_kv_heads, d), _gen(wl, layer, 5, device), device)
    vn = _randn((S, B, wl.n_kv_heads, d), _gen(wl, layer, 6, device), device)
    for c in _outlier_channels(d):
        kn[..., c] *= wl.outlier_gain
    return q.to(torch.bfloat16), kn.to(torch.bfloat16), vn.to(torch.bfloat16)


def to_numpy_f32(t: torch.Tensor):
    """bf16 tensor -> float32 NumPy array holding the same (bf16-exact) values."""
    return t.detach().to("cpu", torch.float32).numpy()
