"""Seeded synthetic inputs shaped like ISOPO's RL microbatches.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic.  It serves both the HIP path and the CPU oracle (which
otherwise share nothing): both see the very same bytes.

The paper's experiments use rollouts of a language model on a maths dataset
(results section); none of that is available or reproduced here.  Only the
shapes (linear-layer sizes of transformer blocks), the ragged sequence
structure (several rollouts per prompt, variable lengths) and rough value
scales are taken.

A layer problem is
    X      [N, d_in]   activations   (fp32, or bf16 stored as torch.bfloat16)
    Delta  [N, d_out]  output grads
    seq_offsets [B+1]  int32 CSR offsets of the contiguous sequences
    A      [B]         fp32 advantages
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Projection:
    name: str
    d_in: int
    d_out: int
    x_key: str  # projections with the same key read the same activations X


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" | "bf16"
    projections: Tuple[Projection, ...]
    n_seq: int
    length_kind: str                # "fixed" | "uniform" | "lognormal"
    length_args: Tuple[float, ...]
    advantages: str                 # "normal" | "grouped_binary"
    group_size: int = 8
    sigma_x: float = 1.0
    sigma_delta: float = 1e-2
    outlier_frac: float = 0.0
    outlier_scale: float = 20.0
    n_layers: int = 1
    seed: int = 1234


def _block(h: int, kv: int, ffn: int) -> Tuple[Projection, ...]:
    return (
        Projection("q", h, h, "attn_in"),
        Projection("k", h, kv, "attn_in"),
        Projection("v", h, kv, "attn_in"),
        Projection("o", h, h, "attn_out"),
        Projection("gate", h, ffn, "mlp_in"),
        Projection("up", h, ffn, "mlp_in"),
        Projection("down", ffn, h, "mlp_mid"),
    )


# The five configurations the benchmark definition names, in its order.
CONFIGS: Dict[str, Workload] = {
    "config1": Workload(
        name="config1", dtype="f32",
        projections=(Projection("lin", 64, 128, "x"),),
        n_seq=4, length_kind="fixed", length_args=(32,),
        advantages="normal", sigma_delta=1e-2, seed=1235),
    "config2": Workload(
        name="config2", dtype="bf16", projections=_block(1536, 256, 8960),
        n_seq=16, length_kind="uniform", length_args=(256, 1024),
        advantages="grouped_binary", sigma_delta=1e-3, outlier_frac=0.01, seed=1236),
    "config3": Workload(
        name="config3", dtype="bf16", projections=_block(4096, 1024, 14336),
        n_seq=32, length_kind="uniform", length_args=(512, 4096),
        advantages="grouped_binary", sigma_delta=1e-3, outlier_frac=0.01, seed=1237),
    "config4": Workload(
        name="config4", dtype="bf16", projections=_block(1536, 256, 8960),
        n_seq=64, length_kind="fixed", length_args=(2048,),
        advantages="grouped_binary", sigma_delta=1e-3, outlier_frac=0.01,
        n_layers=28, seed=1238),
    "config5": Workload(
        name="config5", dtype="bf16",
        projections=(Projection("gate", 5120, 27648, "mlp_in"),),
        n_seq=256, length_kind="lognormal", length_args=(1024.0, 1.0, 128, 16384),
        advantages="grouped_binary", sigma_delta=1e-3, outlier_frac=0.01, seed=1239),
}


def draw_lengths(w: Workload, n_seq: Optional[int] = None, seed: Optional[int] = None) -> np.ndarray:
    """Sequence lengths on the host, seeded."""
    rng = np.random.default_rng((w.seed if seed is None else seed) + 7919)
    b = w.n_seq if n_seq is None else n_seq
    if w.length_kind == "fixed":
        return np.full(b, int(w.length_args[0]), dtype=np.int64)
    if w.length_kind == "uniform":
        lo, hi = int(w.length_args[0]), int(w.length_args[1])
        return rng.integers(lo, hi + 1, size=b, dtype=np.int64)
    if w.length_kind == "lognormal":
        median, sigma, lo, hi = w.length_args
        t = np.rint(np.exp(np.log(median) + sigma * rng.standard_normal(b)))
        return np.clip(t, lo, hi).astype(np.int64)
    raise ValueError(w.length_kind)


def offsets_from_lengths(lengths) -> np.ndarray:
    off = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=off[1:])
    if off[-1] >= 2 ** 31:
        raise ValueError("token count does not fit int32 offsets")
    return off.astype(np.int32)


def draw_advantages(kind: str, n_seq: int, group_size: int, seed: int) -> np.ndarray:
    """fp32 advantages.  "normal": N(0,1) standardised over the batch.
    "grouped_binary": binary rewards standardised within each prompt group,
    A = (r - mean_g) / (std_g + 1e-6) with the population std; a group whose
    rewards are all equal is redrawn (it would carry no signal)."""
    rng = np.random.default_rng(seed + 104729)
    if kind == "normal":
        a = rng.standard_normal(n_seq)
        if n_seq > 1:
            a = (a - a.mean()) / a.std()
        return a.astype(np.float32)
    if kind == "grouped_binary":
        a = np.zeros(n_seq, dtype=np.float64)
        for g0 in range(0, n_seq, group_size):
            g1 = min(n_seq, g0 + group_size)
            if g1 - g0 < 2:
                a[g0:g1] = 1.0
                continue
            while True:
                r = (rng.random(g1 - g0) < 0.5).astype(np.float64)
                if r.min() != r.max():
                    break
            a[g0:g1] = (r - r.mean()) / (r.std() + 1e-6)
        return a.astype(np.float32)
    raise ValueError(kind)


def _torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def _normal(shape, sigma: float, gen: torch.Generator, device) -> torch.Tensor:
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * sigma


def draw_matrix(n: int, d: int, sigma: float, dtype: str, seed: int, device="cpu",
                outlier_frac: float = 0.0, outlier_scale: float = 20.0,
                group_of_token: Optional[torch.Tensor] = None, rho: float = 0.0) -> torch.Tensor:
    """[n, d] iid N(0, sigma^2); a fixed random `outlier_frac` of the channels
    is scaled by `outlier_scale`; with rho > 0 every token also gets rho times
    a vector shared by its prompt group (rollouts of one prompt correlate)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    m = _normal((n, d), sigma, gen, device)
    if rho > 0.0 and group_of_token is not None:
        n_groups = int(group_of_token.max().item()) + 1
        shared = _normal((n_groups, d), sigma, gen, device)
        m += rho * shared[group_of_token.to(device)]
    if outlier_frac > 0.0:
        n_out = max(1, int(round(outlier_frac * d)))
        ch = torch.randperm(d, generator=gen, device=device)[:n_out]
        m[:, ch] *= outlier_scale
    return m.to(_torch_dtype(dtype)).contiguous()


@dataclass
class LayerProblem:
    name: str
    dtype: str
    X: torch.Tensor
    Delta: torch.Tensor
    seq_offsets: np.ndarray          # int32 [B+1], host
    A: np.ndarray                    # fp32 [B], host
    d_in: int
    d_out: int

    @property
    def n_seq(self) -> int:
        return len(self.seq_offsets) - 1

    @property
    def n_tokens(self) -> int:
        return int(self.seq_offsets[-1])


def make_layer(w: Workload, proj: Projection, lengths=None, device="cpu", layer: int = 0,
               rho: float = 0.0, x_cache: Optional[dict] = None, n_seq: Optional[int] = None) -> LayerProblem:
    """One projection's problem.  Projections sharing `x_key` get the same X
    (pass the same `x_cache` dict); every projection has its own Delta."""
    if lengths is None:
        lengths = draw_lengths(w, n_seq=n_seq)
    off = offsets_from_lengths(lengths)
    b = len(lengths)
    n = int(off[-1])
    base = w.seed * 1000 + layer * 37
    groups = torch.from_numpy(np.repeat(np.arange(b) // w.group_size, np.asarray(lengths)))
    key = (proj.x_key, layer)
    if x_cache is not None and key in x_cache:
        X = x_cache[key]
    else:
        x_seed = base + sum(ord(ch) for ch in proj.x_key)
        X = draw_matrix(n, proj.d_in, w.sigma_x, w.dtype, x_seed, device,
                        w.outlier_frac, w.outlier_scale, groups, rho)
        if x_cache is not None:
            x_cache[key] = X
    d_seed = base + 500 + sum(ord(ch) * (i + 1) for i, ch in enumerate(proj.name))
    Delta = draw_matrix(n, proj.d_out, w.sigma_delta, w.dtype, d_seed, device, 0.0, 1.0, groups, rho)
    A = draw_advantages(w.advantages, b, w.group_size, w.seed + layer)
    return LayerProblem(f"{w.name}/{proj.name}", w.dtype, X, Delta, off, A, proj.d_in, proj.d_out)


def make_block(w: Workload, device="cpu", layer: int = 0, rho: float = 0.0,
               lengths=None, n_seq: Optional[int] = None) -> List[LayerProblem]:
    if lengths is None:
        lengths = draw_lengths(w, n_seq=n_seq)
    cache: dict = {}
    return [make_layer(w, p, lengths, device, layer, rho, cache) for p in w.projections]


def custom_layer(d_in: int, d_out: int, lengths, dtype: str = "f32", seed: int = 0, device="cpu",
                 sigma_x: float = 1.0, sigma_delta: float = 1e-2, rho: float = 0.0,
                 group_size: int = 8, advantages: str = "normal") -> LayerProblem:
    """A free-form single layer for edge-case tests."""
    w = Workload(name="custom", dtype=dtype, projections=(Projection("lin", d_in, d_out, "x"),),
                 n_seq=len(lengths), length_kind="fixed", length_args=(0,), advantages=advantages,
                 group_size=group_size, sigma_x=sigma_x, sigma_delta=sigma_delta, seed=seed)
    return make_layer(w, w.projections[0], np.asarray(lengths, dtype=np.int64), device, 0, rho)


def to_oracle(t: torch.Tensor) -> np.ndarray:
    """The exact bytes of a tensor as a numpy array the oracle accepts
    (bf16 -> uint16 bit patterns; fp32 stays fp32)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
