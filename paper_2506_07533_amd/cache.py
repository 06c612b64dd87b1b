"""Host-side bookkeeping of a mixed-precision KV cache built on the three library calls.

Nothing here computes: the classes own the device buffers (torch tensors), keep the counters
(packed chunks, residual length) and decide WHEN the library is called:

* prefill: route every full chunk (Eq. (1)-(2), Sec. 3.2) and pack it; the residual shorter than
  a chunk stays FP16 (Sec. 3.2);
* decode: the new token's K/V row is appended to the FP16 residual; when the residual holds a
  whole chunk it is routed and packed as the next chunk and the residual empties;
* routing sharing (Sec. 3.4): the blocks of a group use the decisions of the group's first
  block, whose router is the only one evaluated;
* routing freezing as the workloads use the word: decisions are taken once and the stored
  tables are reused by every later decode call.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as mq


class LayerCache:
    """Packed K/V of one transformer block: arena + per-chunk tables + FP16 residual."""

    def __init__(self, cfg: mq.Cfg, max_chunks: int, arena_bytes: Optional[int] = None, device="cuda"):
        self.cfg = cfg
        self.BH = cfg.batch * cfg.n_kv_heads
        self.max_chunks = max_chunks
        cap = mq.arena_upper_bound(cfg, self.BH * max_chunks) if arena_bytes is None else arena_bytes
        dev = torch.device(device)
        self.arena = torch.zeros(cap, dtype=torch.uint8, device=dev)
        self.arena_used = torch.zeros(1, dtype=torch.int64, device=dev)
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        cols = (max_chunks + 15) // 16 * 16                   # table rows of whole 16-byte pieces: the pack call then plans one row per workgroup
        self.expert = torch.zeros((self.BH, cols), dtype=torch.uint8, device=dev)
        self.votes = torch.zeros((self.BH, cols, len(cfg.expert_bits)), dtype=torch.int32, device=dev)
        self.chunk_off = torch.zeros((self.BH, cols), dtype=torch.int64, device=dev)
        shape = (cfg.batch, cfg.n_kv_heads, cfg.chunk, cfg.head_dim)
        self.K_tail = torch.zeros(shape, dtype=torch.float16, device=dev)
        self.V_tail = torch.zeros(shape, dtype=torch.float16, device=dev)
        self.n_chunks = 0
        self.n_tail = 0
        self.workspace = torch.zeros(mq.decode_workspace_bytes(cfg, max_chunks), dtype=torch.uint8, device=dev)
        self.planned_chunks = -1                               # n_chunks the plan in the workspace was made for

    # -- routing ---------------------------------------------------------------------------
    def route(self, K: torch.Tensor, c0: int, c1: int, router, token0: int = 0) -> None:
        W1, W2, W3, bias = router
        self.planned_chunks = -1
        mq.route_chunks(self.cfg, K, c0, c1, W1, W2, W3, bias, self.expert, self.votes, token0=token0)

    def share_decisions_from(self, leader: "LayerCache", c0: int, c1: int) -> None:
        """Routing sharing: take the group leader's decisions for chunks [c0, c1)."""
        self.planned_chunks = -1
        self.expert[:, c0:c1].copy_(leader.expert[:, c0:c1])

    # -- packing ---------------------------------------------------------------------------
    def pack(self, K: torch.Tensor, V: torch.Tensor, c0: int, c1: int, token0: int = 0) -> None:
        self.planned_chunks = -1
        mq.quantize_pack(self.cfg, K, V, c0, c1, self.expert, self.arena, self.arena_used, self.chunk_off,
                         self.status, token0=token0)

    def compress_prefill(self, K: torch.Tensor, V: torch.Tensor, router=None, leader: "LayerCache" = None) -> None:
        """K, V: fp16 [B, Hkv, S, D].  Full chunks are routed (or shared) and packed, the rest stays FP16."""
        N = self.cfg.chunk
        S = K.shape[2]
        C, T = S // N, S % N
        assert C <= self.max_chunks
        if leader is None:
            self.route(K, 0, C, router)
        else:
            self.share_decisions_from(leader, 0, C)
        self.pack(K, V, 0, C)
        self.n_chunks, self.n_tail = C, T
        if T:
            self.K_tail[:, :, :T].copy_(K[:, :, C * N:])
            self.V_tail[:, :, :T].copy_(V[:, :, C * N:])

    # -- decode ----------------------------------------------------------------------------
    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, router=None, leader: "LayerCache" = None) -> bool:
        """k_new, v_new: fp16 [B, Hkv, D], the new token.  Returns True when a chunk was flushed."""
        N = self.cfg.chunk
        mq.append_tail(self.cfg, k_new, v_new, self.K_tail, self.V_tail, self.n_tail)
        self.n_tail += 1
        if self.n_tail < N:
            return False
        c = self.n_chunks                                   # the residual is a whole chunk: it becomes chunk c
        assert c < self.max_chunks
        if leader is None:
            self.route(self.K_tail, c, c + 1, router, token0=c * N)
        else:
            self.share_decisions_from(leader, c, c + 1)
        self.pack(self.K_tail, self.V_tail, c, c + 1, token0=c * N)
        self.n_chunks, self.n_tail = c + 1, 0
        return True

    def decode(self, q: torch.Tensor, out: torch.Tensor, softmax_scale: float) -> None:
        """Decode steps reuse the plan of the tables until a chunk is appended (the decisions are made once per chunk)."""
        if self.planned_chunks != self.n_chunks:
            mq.decode_plan(self.cfg, self.expert, self.n_chunks, self.workspace)
            self.planned_chunks = self.n_chunks
        mq.decode_attn(self.cfg, q, self.arena, self.chunk_off, self.expert, self.n_chunks,
                       self.K_tail, self.V_tail, self.n_tail, softmax_scale, out, self.workspace, planned=True)

    def check_status(self) -> None:
        st = int(self.status.item())
        if st != 0:
            raise mq.MoqaeError(st, "quantize_pack (device status)")


class KVStack:
    """A stack of blocks with routing sharing: blocks g*share .. g*share+share-1 form a group
    whose first block routes; the others reuse its decisions (their routers do not exist)."""

    def __init__(self, cfg: mq.Cfg, n_layers: int, share_group: int, max_chunks: int,
                 arena_bytes: Optional[Sequence[int]] = None, device="cuda"):
        self.cfg, self.n_layers, self.share = cfg, n_layers, max(1, share_group)
        self.layers: List[LayerCache] = [
            LayerCache(cfg, max_chunks, None if arena_bytes is None else arena_bytes[l], device) for l in range(n_layers)]

    def leader_of(self, layer: int) -> int:
        return layer - layer % self.share

    def is_leader(self, layer: int) -> bool:
        return layer % self.share == 0

    def compress_prefill(self, layer: int, K, V, routers) -> None:
        lc = self.layers[layer]
        if self.is_leader(layer):
            lc.compress_prefill(K, V, router=routers[layer])
        else:
            lc.compress_prefill(K, V, leader=self.layers[self.leader_of(layer)])

    def append(self, layer: int, k_new, v_new, routers) -> bool:
        lc = self.layers[layer]
        if self.is_leader(layer):
            return lc.append(k_new, v_new, router=routers[layer])
        return lc.append(k_new, v_new, leader=self.layers[self.leader_of(layer)])
