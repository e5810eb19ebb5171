"""Seeded synthetic inputs for the STILL hybrid-attention forward path.

This module holds no arithmetic of the method itself: it only draws random
tensors with the shapes and value distributions of the benchmark workloads and
rounds them to the storage dtype.  Both the CPU oracle's tests and the HIP path
consume exactly the same rounded values, so input rounding is never part of an
error budget.

The tensors stand in for the post-RoPE q/k/v of one Llama-style attention layer
(the paper's efficiency section names only sequence lengths, no dataset).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 260202180


@dataclass(frozen=True)
class Workload:
    """One operator problem: shapes, routing hyper-parameters and dtype."""

    name: str
    B: int
    N: int
    Hq: int
    Hkv: int
    d: int
    C: int          # chunk size
    W: int          # saliency window (keys, inclusive of the token itself)
    lam: int        # tokens kept per full chunk
    dtype: str      # "f32" | "bf16"
    heavy_frac: float = 0.0   # fraction of positions whose key row is scaled by heavy_mult
    heavy_mult: float = 8.0
    d_f: int = 0    # NP-Map inner width (0 => d)
    eps: float = 1e-6
    decode_steps: int = 0
    max_retained: int = 0     # budget on the retained tokens per (sequence, head); 0 => none
    budget_policy: int = 0    # with a budget: 0 = stop adding, 1 = evict the lowest score
    shared_selection: bool = False   # variant: the heads of one kv head rank by their summed score

    @property
    def df(self) -> int:
        return self.d_f if self.d_f else self.d

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    @property
    def seed(self) -> int:
        return BASE_SEED + {"c1": 1, "c2": 2, "c3": 3, "c4": 4, "c5": 5, "c6": 6}.get(self.name, 99)


CONFIGS: Dict[str, Workload] = {
    # tiny fp32 correctness case
    "c1": Workload("c1", B=1, N=1024, Hq=2, Hkv=2, d=64, C=64, W=64, lam=16, dtype="f32"),
    # Llama-3.2-1B-shaped layer
    "c2": Workload("c2", B=4, N=4096, Hq=32, Hkv=8, d=64, C=64, W=64, lam=16, dtype="bf16"),
    # Llama-3-8B-shaped layer
    "c3": Workload("c3", B=2, N=8192, Hq=32, Hkv=8, d=128, C=64, W=128, lam=16, dtype="bf16"),
    # long-context 8B-shaped layer with heavy-hitter keys
    "c4": Workload("c4", B=1, N=32768, Hq=32, Hkv=8, d=128, C=128, W=128, lam=16, dtype="bf16",
                   heavy_frac=0.01),
    # decode at the 8B shape: 64 sequences with a 32K prefilled context each
    "c5": Workload("c5", B=64, N=32768, Hq=32, Hkv=8, d=128, C=128, W=128, lam=16, dtype="bf16",
                   heavy_frac=0.01, decode_steps=128),
    # training shape: the paper trains on sequences of 1024 tokens (Sec. 4.1); 8B-shaped layer, 16 sequences
    "c6": Workload("c6", B=16, N=1024, Hq=32, Hkv=8, d=128, C=64, W=128, lam=16, dtype="bf16"),
}


def workload(name: str, **overrides) -> Workload:
    return replace(CONFIGS[name], **overrides)


# ----------------------------------------------------------------------------
# bf16 storage helpers (bit manipulation only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Value of x after storage in `dtype`, returned as float32 (exactly representable)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------

def make_inputs(w: Workload, seed: Optional[int] = None, with_gate: bool = False,
                n_tokens: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw one problem.  All arrays are float32 holding dtype-rounded values.

    q [B,N,Hq,d]; k,v [B,N,Hkv,d]; Wq,Wk [Hq,d,d_f]; g [B,N,Hq,d] (optional, in (0,1)).
    Draw order is fixed: channel scales, Q, K, V, heavy-hitter positions, Wq, Wk, gate.
    `n_tokens` overrides the sequence length (prefill + decode tokens in one draw).
    """
    rng = np.random.default_rng(w.seed if seed is None else seed)
    N = w.N if n_tokens is None else n_tokens
    B, Hq, Hkv, d, df = w.B, w.Hq, w.Hkv, w.d, w.df
    sq = np.exp(0.5 * rng.standard_normal((Hq, d))).astype(np.float32)
    sk = np.exp(0.5 * rng.standard_normal((Hkv, d))).astype(np.float32)
    sv = np.exp(0.5 * rng.standard_normal((Hkv, d))).astype(np.float32)
    q = rng.standard_normal((B, N, Hq, d), dtype=np.float32) * sq
    k = rng.standard_normal((B, N, Hkv, d), dtype=np.float32) * sk
    v = rng.standard_normal((B, N, Hkv, d), dtype=np.float32) * sv
    heavy = np.zeros((B, 0), dtype=np.int64)
    if w.heavy_frac > 0.0:
        n_heavy = int(w.heavy_frac * N)
        heavy = np.stack([np.sort(rng.choice(N, size=n_heavy, replace=False)) for _ in range(B)])
        for b in range(B):
            k[b, heavy[b]] *= np.float32(w.heavy_mult)
    std = 1.0 / np.sqrt(d)
    Wq = (rng.standard_normal((Hq, d, df)) * std).astype(np.float32)
    Wk = (rng.standard_normal((Hq, d, df)) * std).astype(np.float32)
    out = {
        "q": round_to_dtype(q, w.dtype), "k": round_to_dtype(k, w.dtype),
        "v": round_to_dtype(v, w.dtype), "Wq": round_to_dtype(Wq, w.dtype),
        "Wk": round_to_dtype(Wk, w.dtype), "heavy": heavy,
    }
    if with_gate:
        g = 1.0 / (1.0 + np.exp(-rng.standard_normal((B, N, Hq, d), dtype=np.float32)))
        out["g"] = round_to_dtype(g, w.dtype)
    return out


def kv_head_map(w: Workload) -> np.ndarray:
    """Default GQA map: q-head h reads kv-head h // (Hq / Hkv)."""
    return (np.arange(w.Hq) // (w.Hq // w.Hkv)).astype(np.int32)


def to_torch(x: np.ndarray, dtype: str, device: str = "cuda"):
    """Upload a float32 array holding dtype-rounded values as a torch tensor of that dtype."""
    import torch

    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)
    bits = f32_to_bf16_bits(x).view(np.int16)
    return torch.from_numpy(bits).to(device).view(torch.bfloat16)


def from_torch(t) -> np.ndarray:
    """Download a torch tensor (f32 or bf16) to float32 numpy."""
    import torch

    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return bf16_bits_to_f32(bits)
    return t.detach().cpu().numpy()
