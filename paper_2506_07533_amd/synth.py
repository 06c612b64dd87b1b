"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors; it contains none of the method's
arithmetic (no router, no quantiser, no attention), so the CPU oracle's tests
and the GPU path can both be fed from it without sharing any code of the
method itself.

Stand-ins (the paper evaluates Llama / Mistral KV caches on WikiText2 and
LongBench, Sec. 4.1; neither weights nor datasets are available here):
  V ~ N(0,1); K ~ N(0,1) with four channels per KV head (fixed over tokens)
  scaled by 10 -- the outlier-channel structure of key caches that KIVI
  reports (Sec. 2.2, "KV Cache Optimization"); q ~ N(0,1);
  router weights ~ N(0, 0.02).
For a prescribed expert mix (trained routers are not available) a class is
planted per chunk: its key rows get a mean shift along one of M fixed
orthonormal directions and the router weights point along those directions.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    seq: int                      # cached tokens per sequence
    chunk: int
    group: int
    head_dim: int = 128
    expert_bits: Tuple[int, ...] = (2, 4, 8, 16)
    freeze_chunks: int = 1
    mix: Optional[Tuple[float, ...]] = None   # planted share of each expert, or None = unplanted
    seed: int = 0
    n_layers: int = 1
    share_group: int = 1          # routing sharing: layers per group
    decode_steps: int = 1

    @property
    def n_chunks(self) -> int:
        return self.seq // self.chunk

    @property
    def n_tail(self) -> int:
        return self.seq % self.chunk


MIX = (0.60, 0.30, 0.05, 0.05)

# The five workloads of the benchmark plan.
WORKLOADS = {
    "tiny":       Workload("tiny", 1, 8, 8, 2048, 64, 32, seed=0),
    "llama7b_32k": Workload("llama7b_32k", 1, 32, 32, 32768, 128, 64, seed=2),
    "llama13b_128k": Workload("llama13b_128k", 1, 40, 40, 131072, 128, 64, mix=MIX, seed=3),
    "gqa8b_128k": Workload("gqa8b_128k", 4, 32, 8, 131072, 256, 64, mix=MIX, seed=4),
    "stack32_32k": Workload("stack32_32k", 16, 32, 32, 32768, 128, 64, mix=MIX, seed=5,
                            n_layers=32, share_group=4, decode_steps=64),
}


def outlier_channels(rng: np.random.Generator, n_units: int, D: int, n_out: int = 4) -> np.ndarray:
    """[n_units, n_out] channel indices, drawn once per (sequence, KV head)."""
    return np.stack([rng.choice(D, size=n_out, replace=False) for _ in range(n_units)])


def planted_directions(M: int, D: int, seed: int) -> np.ndarray:
    """[M, D] orthonormal rows."""
    rng = np.random.default_rng([seed, 77])
    qmat, _ = np.linalg.qr(rng.standard_normal((D, M)))
    return np.ascontiguousarray(qmat.T.astype(np.float32))


def make_router(D: int, M: int, seed: int, std: float = 0.02,
                directions: Optional[np.ndarray] = None, gamma: float = 1.0):
    """Router weights W1, W2 [D, M] and W3 [M, M] as fp16.

    Unplanted: all three ~ N(0, std).  Planted: W1 = W2 = gamma * directions^T
    + N(0, std), W3 = I + N(0, std)."""
    rng = np.random.default_rng([seed, 11])
    W1 = rng.standard_normal((D, M)).astype(np.float32) * std
    W2 = rng.standard_normal((D, M)).astype(np.float32) * std
    W3 = rng.standard_normal((M, M)).astype(np.float32) * std
    if directions is not None:
        W1 += gamma * directions.T
        W2 += gamma * directions.T
        W3 += np.eye(M, dtype=np.float32)
    return W1.astype(np.float16), W2.astype(np.float16), W3.astype(np.float16)


def make_q(B: int, Hq: int, D: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 23])
    return rng.standard_normal((B, Hq, D), dtype=np.float32).astype(np.float16)


def make_classes(n_units: int, n_chunks: int, mix: Sequence[float], seed: int) -> np.ndarray:
    """[n_units, n_chunks] planted class of every chunk, i.i.d. from `mix`."""
    rng = np.random.default_rng([seed, 31])
    return rng.choice(len(mix), size=(n_units, n_chunks), p=np.asarray(mix, np.float64)).astype(np.uint8)


def make_kv(B: int, Hkv: int, S: int, D: int, seed: int, chunk: int = 0,
            classes: Optional[np.ndarray] = None, directions: Optional[np.ndarray] = None,
            mu: float = 6.0, outlier_scale: float = 10.0):
    """K, V fp16 [B, Hkv, S, D].  With `classes` ([B*Hkv, C]) and `directions`
    ([M, D]) the rows of chunk c of unit u are shifted by mu * directions[classes[u, c]]."""
    K = np.empty((B, Hkv, S, D), np.float16)
    V = np.empty((B, Hkv, S, D), np.float16)
    chans = outlier_channels(np.random.default_rng([seed, 5]), B * Hkv, D)
    for u in range(B * Hkv):
        rng = np.random.default_rng([seed, 1000 + u])
        k = rng.standard_normal((S, D), dtype=np.float32)
        k[:, chans[u]] *= outlier_scale
        if classes is not None:
            C = classes.shape[1]
            shift = mu * directions[classes[u]]                     # [C, D]
            k[: C * chunk].reshape(C, chunk, D)[...] += shift[:, None, :]
        K[u // Hkv, u % Hkv] = k.astype(np.float16)
        V[u // Hkv, u % Hkv] = rng.standard_normal((S, D), dtype=np.float32).astype(np.float16)
    return K, V


def make_workload(w: Workload, layer: int = 0, seq: Optional[int] = None):
    """All host inputs of one layer of workload `w` as a dict of numpy arrays."""
    S = w.seq if seq is None else seq
    M = len(w.expert_bits)
    seed = w.seed * 1000 + layer
    C = S // w.chunk
    classes = dirs = None
    if w.mix is not None:
        dirs = planted_directions(M, w.head_dim, w.seed)
        classes = make_classes(w.batch * w.n_kv_heads, C, w.mix, seed)
    K, V = make_kv(w.batch, w.n_kv_heads, S, w.head_dim, seed, w.chunk, classes, dirs)
    W1, W2, W3 = make_router(w.head_dim, M, w.seed, directions=dirs)
    q = make_q(w.batch, w.n_q_heads, w.head_dim, seed)
    return dict(K=K, V=V, W1=W1, W2=W2, W3=W3, q=q, classes=classes)


def make_layer_device(w: Workload, layer: int, device, seq: Optional[int] = None):
    """One layer of workload `w` drawn directly on the GPU (for layers too large to stage through
    the host).  Same recipe as make_workload; the bits differ from the host generator's, parity
    tests copy back the slices they check.  Returns torch tensors."""
    import torch
    S = w.seq if seq is None else seq
    M = len(w.expert_bits)
    seed = w.seed * 1000 + layer
    B, H, D, N = w.batch, w.n_kv_heads, w.head_dim, w.chunk
    C = S // N
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    K = torch.randn((B, H, S, D), generator=g, device=device, dtype=torch.float16)
    V = torch.randn((B, H, S, D), generator=g, device=device, dtype=torch.float16)
    chans = outlier_channels(np.random.default_rng([seed, 5]), B * H, D)
    scale = np.ones((B * H, D), np.float32)
    np.put_along_axis(scale, chans, 10.0, axis=1)
    K.mul_(torch.from_numpy(scale).to(device=device, dtype=torch.float16).view(B, H, 1, D))
    classes = dirs = None
    if w.mix is not None:
        dirs = planted_directions(M, D, w.seed)
        classes = make_classes(B * H, C, w.mix, seed)
        shift = torch.from_numpy(6.0 * dirs[classes]).to(device=device, dtype=torch.float16)     # [B*H, C, D]
        K[:, :, : C * N].view(B, H, C, N, D).add_(shift.view(B, H, C, 1, D))
    W1, W2, W3 = make_router(D, M, w.seed, directions=dirs)
    q = make_q(B, w.n_q_heads, D, seed)
    return dict(K=K, V=V, W1=torch.from_numpy(W1).to(device), W2=torch.from_numpy(W2).to(device),
                W3=torch.from_numpy(W3).to(device), q=torch.from_numpy(q).to(device), classes=classes)
