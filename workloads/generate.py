"""Seeded synthetic inputs for the StructKV scoring / selection / gather path.

This module only *draws* inputs (window queries, keys, values, hub positions).
It contains none of the method's arithmetic (no softmax, no in-degree, no
selection): both the CPU oracle's tests and the HIP path's tests/bench take
their inputs from here, and nothing else is shared between the two.

The shapes stand in for a LLaMA-3-8B-shaped prefill (the paper's Sec. 4.1
models at 8K-128K contexts); the paper's datasets and weights are not used.

Recipe (per layer, per tensor, independent seeded streams):
  * Q_win, K, V ~ N(0, 1) i.i.d. (torch.Generator seeded by a splitmix64 mix of
    (base seed, workload name, layer, tensor id)).
  * optional AR(1) structure along the token axis for K
    (k_j = rho k_{j-1} + sqrt(1-rho^2) eps_j, unit marginal variance).
  * planted hub keys: at hub positions (stratified over [0, n-w)), in the layers
    where the hub is active, k_hub = eps + 4 sqrt(d) u_g, with u_g the unit
    vector of the mean of the KV group's window queries ("K scaled x4 along the
    mean query direction": a key ~4x the typical norm, aligned with the queries).
    hub_mode "all": active in every layer; "half": active in a seeded random
    half of the layers, an ordinary N(0,1) key ("dormant") in the others.
  * everything is rounded to the workload dtype (fp32 or bf16) last.
"""
from __future__ import annotations

import dataclasses
import math
import zlib
from typing import List, Sequence, Tuple

import numpy as np
import torch

_MASK64 = (1 << 64) - 1


def _splitmix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _MASK64
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_lens: Tuple[int, ...]      # one entry per sequence of the (ragged) batch
    window: int
    dtype: str                     # "f32" | "bf16"
    k_per_seq: Tuple[int, ...]     # top-k budget per sequence (window is kept on top)
    n_hubs: int                    # planted hubs per sequence
    hub_mode: str = "all"          # "all" | "half"
    ar1_rho: float = 0.0
    seed: int = 6746
    lam: float = 0.9               # decay used by the sweep (paper Sec. 4.1 default)

    @property
    def batch(self) -> int:
        return len(self.seq_lens)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seq_lens))

    @property
    def cu_seqlens(self) -> List[int]:
        cu = [0]
        for n in self.seq_lens:
            cu.append(cu[-1] + int(n))
        return cu

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]

    @property
    def elem_bytes(self) -> int:
        return {"f32": 4, "bf16": 2}[self.dtype]

    def stream_seed(self, layer: int, tensor_id: int) -> int:
        s = _splitmix64(self.seed & _MASK64)
        for v in (zlib.crc32(self.name.encode()), layer & 0xFFFFFFFF, tensor_id):
            s = _splitmix64(s ^ v)
        return s & ((1 << 63) - 1)


def _ragged_lengths(seed: int, batch: int, lo: int, hi: int) -> Tuple[int, ...]:
    out = []
    s = seed
    for _ in range(batch):
        s = _splitmix64(s)
        out.append(lo + s % (hi - lo + 1))
    return tuple(out)


def _c5_lengths() -> Tuple[int, ...]:
    return _ragged_lengths(6746 * 5, 8, 16384, 131072)


# The five benchmark configurations (C1..C5) plus small parity-test shapes.
WORKLOADS = {}


def _register(w: Workload) -> Workload:
    WORKLOADS[w.name] = w
    return w


C1_TINY = _register(Workload("c1_tiny", 4, 8, 8, 64, (1024,), 32, "f32", (128,), 4, "all"))
C2_32K = _register(Workload("c2_llama8b_32k", 32, 32, 8, 128, (32768,), 32, "bf16", (2048,), 64, "half"))
C3_128K = _register(Workload("c3_llama8b_128k", 32, 32, 8, 128, (131072,), 64, "bf16", (4096,), 256, "half",
                             ar1_rho=0.9))
C4_1M = _register(Workload("c4_llama8b_1m", 32, 32, 8, 128, (1048576,), 64, "bf16", (16384,), 1024, "half"))
_c5 = _c5_lengths()
C5_RAGGED = _register(Workload("c5_ragged_batch8", 32, 32, 8, 128, _c5, 32, "bf16",
                               tuple(int(0.05 * n) for n in _c5), 32, "half"))

# The paper's own operating point (Sec. 4.1 / 4.6: LLaMA-3.1-8B, 32K-token prefill, observation window 8, 10 % KV
# budget): not one of the five benchmark configurations, kept as context for the ~35 ms the paper reports there.
P_32K_W8 = _register(Workload("p_llama8b_32k_w8", 32, 32, 8, 128, (32768,), 8, "bf16", (3276,), 64, "half"))

# Small shapes for element-by-element parity: several key tiles + a ragged tail.
S_BF16 = _register(Workload("s_bf16_gqa4", 3, 8, 2, 128, (2437,), 32, "bf16", (100,), 6, "half"))
S_BF16_W64 = _register(Workload("s_bf16_w64", 2, 8, 2, 128, (3001,), 64, "bf16", (150,), 4, "all", ar1_rho=0.9))
S_BF16_D64 = _register(Workload("s_bf16_d64", 2, 4, 4, 64, (1111,), 32, "bf16", (64,), 4, "all"))
S_BF16_RAGGED = _register(Workload("s_bf16_ragged", 2, 8, 2, 128, (700, 33, 1500, 64), 32, "bf16",
                                   (35, 1, 75, 3), 2, "all"))
# KV groups above 128 query rows that are not four full 64-row chunks: 3 x 64 = 192 rows (one idle wave),
# 4 x 40 = 160 rows (a partly padded chunk), 8 x 64 = 512 rows (two workgroups per key chunk); d = 64 at 256 rows
S_BF16_R192 = _register(Workload("s_bf16_r192", 2, 6, 2, 128, (1300, 90), 64, "bf16", (60, 4), 3, "all"))
S_BF16_R160 = _register(Workload("s_bf16_r160", 2, 8, 2, 128, (999,), 40, "bf16", (50,), 3, "all"))
S_BF16_R512 = _register(Workload("s_bf16_r512", 2, 16, 2, 128, (2100,), 64, "bf16", (100,), 3, "all"))
S_BF16_D64_R256 = _register(Workload("s_bf16_d64_r256", 2, 8, 2, 64, (1500,), 64, "bf16", (70,), 3, "all"))
# small KV groups on the bf16 path: the paper's window of 8 (4 x 8 = 32 rows, one 32-row wave) and 64 rows
S_BF16_W8 = _register(Workload("s_bf16_w8", 2, 8, 2, 128, (1234, 77), 8, "bf16", (60, 5), 3, "all"))
S_BF16_R64 = _register(Workload("s_bf16_r64", 2, 4, 2, 128, (1800,), 32, "bf16", (90,), 3, "all"))
# 65..128 rows run as four waves of 32 rows: 3 x 32 = 96 rows (one idle wave) and 5 x 24 = 120 rows (heads straddle waves)
S_BF16_R96 = _register(Workload("s_bf16_r96", 2, 6, 2, 128, (1700, 45), 32, "bf16", (80, 2), 3, "all"))
# 6 heads x 32 rows = 192 rows in 64-row waves: each of a wave's two 32-row blocks is one head's window
S_BF16_R192_W32 = _register(Workload("s_bf16_r192_w32", 2, 12, 2, 128, (1400, 200), 32, "bf16", (70, 10), 3, "all"))
S_BF16_R120 = _register(Workload("s_bf16_r120", 2, 10, 2, 64, (1203,), 24, "bf16", (60,), 3, "all"))
S_F32_W8 = _register(Workload("s_f32_w8", 2, 4, 2, 64, (777,), 8, "f32", (50,), 3, "all"))
S_F32_RAGGED = _register(Workload("s_f32_ragged", 2, 8, 8, 64, (300, 40, 513), 32, "f32", (15, 2, 25), 2, "all"))


def hub_positions(wl: Workload) -> List[List[int]]:
    """Sequence-local hub positions, stratified over [0, n_b - w)."""
    out = []
    for b, n in enumerate(wl.seq_lens):
        span = n - wl.window
        pos: List[int] = []
        if wl.n_hubs > 0 and span >= wl.n_hubs:
            s = wl.stream_seed(-1, 100 + b)
            for i in range(wl.n_hubs):
                s = _splitmix64(s)
                u = (s >> 11) / float(1 << 53)
                lo = (i * span) // wl.n_hubs
                hi = ((i + 1) * span) // wl.n_hubs
                pos.append(min(hi - 1, lo + int(u * (hi - lo))))
        out.append(pos)
    return out


def hub_active(wl: Workload, layer: int) -> List[List[bool]]:
    """active[b][i]: is hub i of sequence b a hub (True) or dormant (False) in this layer."""
    pos = hub_positions(wl)
    out = []
    for b in range(wl.batch):
        row = []
        for i in range(len(pos[b])):
            if wl.hub_mode == "all":
                row.append(True)
                continue
            # seeded random half of the layers: rank the layers by a hash, keep the lower half
            keys = [(_splitmix64(wl.stream_seed(-2, 1000 * b + i) ^ l), l) for l in range(wl.n_layers)]
            keys.sort()
            active_layers = {l for _, l in keys[: wl.n_layers // 2]}
            row.append(layer in active_layers)
        out.append(row)
    return out


@dataclasses.dataclass
class LayerInputs:
    q_win: torch.Tensor   # [B, H_q, w, d]
    k: torch.Tensor       # [G, total_tokens, d]
    v: torch.Tensor       # [G, total_tokens, d]


def _randn(shape: Sequence[int], seed: int, device) -> torch.Tensor:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn(*shape, generator=g, device=device, dtype=torch.float32)


def _ar1_along_tokens(eps: torch.Tensor, rho: float, cu: List[int]) -> torch.Tensor:
    """y_j = rho y_{j-1} + sqrt(1-rho^2) eps_j within each sequence (y_0 = eps_0), tokens on dim 1."""
    out = torch.empty_like(eps)
    c = math.sqrt(1.0 - rho * rho)
    for b in range(len(cu) - 1):
        lo, hi = cu[b], cu[b + 1]
        if hi == lo:
            continue
        y = eps[:, lo:hi, :] * c
        y[:, 0, :] = eps[:, lo, :]
        s = 1
        while s < hi - lo and rho ** s > 1e-20:
            y2 = y.clone()
            y2[:, s:, :] += (rho ** s) * y[:, :-s, :]
            y = y2
            s *= 2
        out[:, lo:hi, :] = y
    return out


def make_layer(wl: Workload, layer: int, device="cpu") -> LayerInputs:
    """Draw one layer's Q_win, K, V on `device`; deterministic per (workload, layer, device type)."""
    B, Hq, G, d, w = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window
    T = wl.total_tokens
    gs = Hq // G
    dt = wl.torch_dtype
    q = _randn((B, Hq, w, d), wl.stream_seed(layer, 1), device).to(dt)
    k = _randn((G, T, d), wl.stream_seed(layer, 2), device)
    if wl.ar1_rho:
        k = _ar1_along_tokens(k, wl.ar1_rho, wl.cu_seqlens)
    pos = hub_positions(wl)
    act = hub_active(wl, layer)
    cu = wl.cu_seqlens
    for b in range(B):
        rows = [cu[b] + p for p, a in zip(pos[b], act[b]) if a]
        if not rows:
            continue
        qm = q[b].to(torch.float64).reshape(G, gs * w, d).mean(dim=1)          # [G, d]
        u = qm / qm.norm(dim=1, keepdim=True).clamp_min(1e-30)
        idx = torch.tensor(rows, device=device, dtype=torch.long)
        k[:, idx, :] += (4.0 * math.sqrt(d)) * u.to(torch.float32)[:, None, :]
    k = k.to(dt)
    v = _randn((G, T, d), wl.stream_seed(layer, 3), device).to(dt)
    return LayerInputs(q, k, v)


def to_oracle_array(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> the host array the CPU oracle takes, bit for bit: fp32 -> float32 ndarray,
    bf16 -> uint16 ndarray of the same bit patterns (a conversion, no arithmetic)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    assert t.dtype == torch.float32
    return t.numpy()
