"""Thin ctypes binding of libmoqae.so: argument marshalling only.

Every function takes torch tensors that live on the GPU (or raw device
pointers) and enqueues the library call on torch's current stream.  There is
no CPU fallback: if the shared library is missing, importing fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoqae.so")

OK, E_INVAL, E_WORKSPACE, E_ARENA, E_HIP = 0, -1, -2, -3, -4


class MoqaeError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class _Cfg(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("chunk", C.c_int32), ("group", C.c_int32),
                ("n_experts", C.c_int32), ("expert_bits", C.c_int32 * 8),
                ("freeze_chunks", C.c_int32), ("k_per_channel", C.c_int32)]


@dataclass
class Cfg:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    chunk: int = 128
    group: int = 64
    expert_bits: Sequence[int] = field(default_factory=lambda: (2, 4, 8, 16))
    freeze_chunks: int = 1
    k_per_channel: int = 0

    def c(self) -> _Cfg:
        bits = list(self.expert_bits) + [0] * (8 - len(self.expert_bits))
        return _Cfg(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.chunk,
                    self.group, len(self.expert_bits), (C.c_int32 * 8)(*bits), self.freeze_chunks, self.k_per_channel)


class _PoolCfg(C.Structure):
    _fields_ = [("n_pages", C.c_int32 * 8)]


def _pc(n_pages: Sequence[int]) -> _PoolCfg:
    return _PoolCfg((C.c_int32 * 8)(*(list(n_pages) + [0] * (8 - len(n_pages)))))


_lib = None
EXPORTS = ["moqae_route_chunks", "moqae_quantize_pack", "moqae_decode_attn", "moqae_chunk_block_bytes",
           "moqae_arena_upper_bound", "moqae_decode_workspace_bytes", "moqae_strerror", "moqae_abi_version",
           "moqae_decode_attn_ragged", "moqae_decode_workspace_bytes_ragged",
           "moqae_decode_plan", "moqae_decode_attn_planned", "moqae_append_tail",
           "moqae_decode_attn_static", "moqae_static_scratch_bytes",
           "moqae_pool_page_bytes", "moqae_pool_base", "moqae_pool_arena_bytes", "moqae_pool_state_bytes",
           "moqae_pool_init", "moqae_route_pack_paged", "moqae_pool_release", "moqae_pool_free_pages",
           "moqae_router_loss_grad", "moqae_decode_attn_multi", "moqae_decode_workspace_bytes_multi"]
# measurement aids of include/moqae_bench.h (bench.py only)
BENCH_EXPORTS = ["moqae_bench_time_decode_kernel", "moqae_bench_stream_read", "moqae_bench_stream_sink_words"]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2506_07533_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(_LIB_PATH)
        vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
        L.moqae_route_chunks.restype = C.c_int
        L.moqae_route_chunks.argtypes = [C.POINTER(_Cfg), vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, i64, vp, vp]
        L.moqae_quantize_pack.restype = C.c_int
        L.moqae_quantize_pack.argtypes = [C.POINTER(_Cfg), vp, vp, i64, i64, i64, i32, i32, vp, i64, vp, u64, vp,
                                          vp, i64, vp, vp]
        L.moqae_decode_attn.restype = C.c_int
        L.moqae_decode_attn.argtypes = [C.POINTER(_Cfg), vp, vp, vp, vp, i64, i32, vp, vp, i32, C.c_float, vp,
                                        vp, u64, vp]
        L.moqae_decode_attn_planned.restype = C.c_int
        L.moqae_decode_attn_planned.argtypes = L.moqae_decode_attn.argtypes
        L.moqae_decode_attn_static.restype = C.c_int
        L.moqae_decode_attn_static.argtypes = [C.POINTER(_Cfg), vp, vp, vp, vp, i64, i32, vp, vp, i32, C.c_float, vp, vp]
        L.moqae_static_scratch_bytes.restype = u64
        L.moqae_static_scratch_bytes.argtypes = []
        pcp = C.POINTER(_PoolCfg)
        L.moqae_pool_page_bytes.restype = u64
        L.moqae_pool_page_bytes.argtypes = [C.POINTER(_Cfg), i32]
        L.moqae_pool_base.restype = u64
        L.moqae_pool_base.argtypes = [C.POINTER(_Cfg), pcp, i32]
        L.moqae_pool_arena_bytes.restype = u64
        L.moqae_pool_arena_bytes.argtypes = [C.POINTER(_Cfg), pcp]
        L.moqae_pool_state_bytes.restype = u64
        L.moqae_pool_state_bytes.argtypes = [C.POINTER(_Cfg), pcp]
        L.moqae_pool_init.restype = C.c_int
        L.moqae_pool_init.argtypes = [C.POINTER(_Cfg), pcp, vp, vp]
        L.moqae_route_pack_paged.restype = C.c_int
        L.moqae_route_pack_paged.argtypes = [C.POINTER(_Cfg), pcp, vp, vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, i64, vp,
                                             vp, vp, vp, i64, vp, vp]
        L.moqae_decode_attn_multi.restype = C.c_int
        L.moqae_decode_attn_multi.argtypes = [C.POINTER(_Cfg), vp, i32, vp, vp, vp, i64, i32, vp, vp, i32, C.c_float, vp, vp, u64, vp]
        L.moqae_decode_workspace_bytes_multi.restype = u64
        L.moqae_decode_workspace_bytes_multi.argtypes = [C.POINTER(_Cfg), i32, i32]
        L.moqae_router_loss_grad.restype = C.c_int
        L.moqae_router_loss_grad.argtypes = [C.POINTER(_Cfg), vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp,
                                             C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_float, vp, vp, vp, vp, vp, vp]
        L.moqae_pool_free_pages.restype = C.c_int
        L.moqae_pool_free_pages.argtypes = [C.POINTER(_Cfg), pcp, vp, vp, vp]
        L.moqae_pool_release.restype = C.c_int
        L.moqae_pool_release.argtypes = [C.POINTER(_Cfg), pcp, vp, i64, vp, i64, i32, i32, i32, i32, vp, vp]
        L.moqae_decode_plan.restype = C.c_int
        L.moqae_decode_plan.argtypes = [C.POINTER(_Cfg), vp, i64, i32, vp, u64, vp]
        L.moqae_append_tail.restype = C.c_int
        L.moqae_append_tail.argtypes = [C.POINTER(_Cfg), vp, vp, vp, vp, i32, vp]
        L.moqae_decode_attn_ragged.restype = C.c_int
        L.moqae_decode_attn_ragged.argtypes = [C.POINTER(_Cfg), vp, vp, vp, vp, i64, vp, i32, vp, vp, vp, C.c_float, vp,
                                               vp, u64, vp]
        L.moqae_decode_workspace_bytes_ragged.restype = u64
        L.moqae_decode_workspace_bytes_ragged.argtypes = [C.POINTER(_Cfg), i32]
        L.moqae_chunk_block_bytes.restype = u64
        L.moqae_chunk_block_bytes.argtypes = [C.POINTER(_Cfg), i32]
        L.moqae_arena_upper_bound.restype = u64
        L.moqae_arena_upper_bound.argtypes = [C.POINTER(_Cfg), i64]
        L.moqae_decode_workspace_bytes.restype = u64
        L.moqae_decode_workspace_bytes.argtypes = [C.POINTER(_Cfg), i32]
        L.moqae_strerror.restype = C.c_char_p
        L.moqae_strerror.argtypes = [C.c_int]
        L.moqae_abi_version.restype = C.c_uint32
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().moqae_strerror(code).decode()


def abi_version() -> int:
    return int(lib().moqae_abi_version())


def chunk_block_bytes(cfg: Cfg, bits: int) -> int:
    return int(lib().moqae_chunk_block_bytes(C.byref(cfg.c()), bits))


def arena_upper_bound(cfg: Cfg, n_chunks_total: int) -> int:
    return int(lib().moqae_arena_upper_bound(C.byref(cfg.c()), n_chunks_total))


def decode_workspace_bytes(cfg: Cfg, n_chunks: int) -> int:
    return int(lib().moqae_decode_workspace_bytes(C.byref(cfg.c()), n_chunks))


def decode_workspace_bytes_ragged(cfg: Cfg, max_chunks: int) -> int:
    return int(lib().moqae_decode_workspace_bytes_ragged(C.byref(cfg.c()), max_chunks))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        raise MoqaeError(rc, what)


def _kv_strides(K: torch.Tensor, cfg: Cfg):
    assert K.is_cuda and K.dtype == torch.float16 and K.dim() == 4 and K.stride(3) == 1
    assert K.shape[0] == cfg.batch and K.shape[1] == cfg.n_kv_heads and K.shape[3] == cfg.head_dim
    return K.stride(0), K.stride(1), K.stride(2)


def route_chunks(cfg: Cfg, K: torch.Tensor, chunk_begin: int, chunk_end: int,
                 W1: torch.Tensor, W2: torch.Tensor, W3: torch.Tensor, bias: Optional[torch.Tensor],
                 expert: torch.Tensor, votes: Optional[torch.Tensor] = None, token0: int = 0) -> None:
    """expert: uint8 [B*Hkv, Ccap]; votes: int32 [B*Hkv, Ccap, M] or None.
    `token0`: K holds tokens token0.. of every sequence (e.g. the FP16 residual buffer when it is
    flushed as chunk token0 / N); the base pointer is shifted so that chunk indices stay absolute."""
    sb, sh, ss = _kv_strides(K, cfg)
    assert K.shape[2] + token0 >= chunk_end * cfg.chunk and chunk_begin * cfg.chunk >= token0
    assert expert.dtype == torch.uint8 and expert.dim() == 2 and expert.is_contiguous() and expert.is_cuda
    if votes is not None:
        assert votes.dtype == torch.int32 and votes.is_contiguous() and votes.shape[:2] == expert.shape
    for w in (W1, W2, W3):
        assert w.is_cuda and w.dtype == torch.float16 and w.is_contiguous()
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.float32 and bias.is_contiguous()
    kptr = C.c_void_p(K.data_ptr() - token0 * ss * 2)
    _check(lib().moqae_route_chunks(C.byref(cfg.c()), kptr, sb, sh, ss, chunk_begin, chunk_end,
                                    _ptr(W1), _ptr(W2), _ptr(W3), _ptr(bias), _ptr(expert), expert.shape[1],
                                    _ptr(votes), _stream()), "moqae_route_chunks")


def quantize_pack(cfg: Cfg, K: torch.Tensor, V: torch.Tensor, chunk_begin: int, chunk_end: int,
                  expert: torch.Tensor, arena: torch.Tensor, arena_used: torch.Tensor,
                  chunk_off: torch.Tensor, status: torch.Tensor, token0: int = 0) -> None:
    """arena: uint8 [capacity]; arena_used: int64 [1]; chunk_off: int64 [B*Hkv, Ccap]; status: int32 [1]."""
    sb, sh, ss = _kv_strides(K, cfg)
    assert _kv_strides(V, cfg) == (sb, sh, ss)
    assert K.shape[2] + token0 >= chunk_end * cfg.chunk and chunk_begin * cfg.chunk >= token0
    assert expert.dtype == torch.uint8 and expert.dim() == 2 and expert.is_contiguous()
    assert chunk_off.dtype == torch.int64 and chunk_off.dim() == 2 and chunk_off.is_contiguous()
    assert arena.dtype == torch.uint8 and arena.is_contiguous() and arena_used.dtype == torch.int64
    assert status.dtype == torch.int32
    shift = token0 * ss * 2
    _check(lib().moqae_quantize_pack(C.byref(cfg.c()), C.c_void_p(K.data_ptr() - shift), C.c_void_p(V.data_ptr() - shift),
                                     sb, sh, ss, chunk_begin, chunk_end, _ptr(expert), expert.shape[1],
                                     _ptr(arena), arena.numel(), _ptr(arena_used), _ptr(chunk_off), chunk_off.shape[1],
                                     _ptr(status), _stream()), "moqae_quantize_pack")


def router_loss_grad(cfg: Cfg, K: torch.Tensor, token_begin: int, token_end: int, W1: torch.Tensor, W2: torch.Tensor,
                     W3: torch.Tensor, bias: Optional[torch.Tensor], nll: torch.Tensor,
                     penalty_model: Optional[Sequence[float]], penalty_mem: Optional[Sequence[float]], lam: float,
                     loss: torch.Tensor, dW1: torch.Tensor, dW2: torch.Tensor, dW3: torch.Tensor,
                     dbias: Optional[torch.Tensor]) -> None:
    """Eq. (3)-(5) and their gradient (moqae_router_loss_grad).  nll: fp32 [B]; loss: fp32 [3]; dW1, dW2: fp32 [D, M];
    dW3: fp32 [M, M]; dbias: fp32 [M] or None; penalties: host sequences of M floats or None (the printed ones)."""
    sb, sh, ss = _kv_strides(K, cfg)
    M = len(cfg.expert_bits)
    assert 0 <= token_begin < token_end <= K.shape[2]
    for w in (W1, W2, W3):
        assert w.is_cuda and w.dtype == torch.float16 and w.is_contiguous()
    assert nll.is_cuda and nll.dtype == torch.float32 and nll.shape == (cfg.batch,)
    for t, shape in ((loss, (3,)), (dW1, (cfg.head_dim, M)), (dW2, (cfg.head_dim, M)), (dW3, (M, M))):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == shape
    if dbias is not None:
        assert dbias.is_cuda and dbias.dtype == torch.float32 and tuple(dbias.shape) == (M,)
    arr = lambda p: None if p is None else (C.c_float * M)(*[float(v) for v in p])
    _check(lib().moqae_router_loss_grad(C.byref(cfg.c()), _ptr(K), sb, sh, ss, token_begin, token_end, _ptr(W1), _ptr(W2), _ptr(W3),
                                        _ptr(bias), _ptr(nll), arr(penalty_model), arr(penalty_mem), float(lam),
                                        _ptr(loss), _ptr(dW1), _ptr(dW2), _ptr(dW3), _ptr(dbias), _stream()),
           "moqae_router_loss_grad")


def pool_page_bytes(cfg: Cfg, expert: int) -> int:
    return int(lib().moqae_pool_page_bytes(C.byref(cfg.c()), expert))


def pool_base(cfg: Cfg, n_pages: Sequence[int], expert: int) -> int:
    return int(lib().moqae_pool_base(C.byref(cfg.c()), C.byref(_pc(n_pages)), expert))


def pool_arena_bytes(cfg: Cfg, n_pages: Sequence[int]) -> int:
    return int(lib().moqae_pool_arena_bytes(C.byref(cfg.c()), C.byref(_pc(n_pages))))


def pool_state_bytes(cfg: Cfg, n_pages: Sequence[int]) -> int:
    return int(lib().moqae_pool_state_bytes(C.byref(cfg.c()), C.byref(_pc(n_pages))))


def pool_init(cfg: Cfg, n_pages: Sequence[int], state: torch.Tensor) -> None:
    """state: int32 / uint8 device tensor of pool_state_bytes() bytes."""
    assert state.is_cuda and state.is_contiguous() and state.numel() * state.element_size() >= pool_state_bytes(cfg, n_pages)
    _check(lib().moqae_pool_init(C.byref(cfg.c()), C.byref(_pc(n_pages)), _ptr(state), _stream()), "moqae_pool_init")


def pool_free_pages(cfg: Cfg, n_pages: Sequence[int], state: torch.Tensor) -> list:
    """Free pages of every pool (synchronises: a test / monitoring aid)."""
    counts = torch.zeros(8, dtype=torch.int32, device=state.device)
    _check(lib().moqae_pool_free_pages(C.byref(cfg.c()), C.byref(_pc(n_pages)), _ptr(state), _ptr(counts), _stream()),
           "moqae_pool_free_pages")
    return [int(v) for v in counts.cpu().tolist()][:len(cfg.expert_bits)]


def route_pack_paged(cfg: Cfg, n_pages: Sequence[int], K: torch.Tensor, V: torch.Tensor, chunk_begin: int, chunk_end: int,
                     router, expert: torch.Tensor, votes: Optional[torch.Tensor], arena: torch.Tensor, state: torch.Tensor,
                     chunk_off: torch.Tensor, status: torch.Tensor, token0: int = 0) -> None:
    """router: (W1, W2, W3, bias or None), or None: `expert` then holds the decisions to use (routing sharing).
    arena: uint8 [pool_arena_bytes]; state: pool state; chunk_off: int64 [B*Hkv, Ccap]; status: int32 [1]."""
    sb, sh, ss = _kv_strides(K, cfg)
    assert _kv_strides(V, cfg) == (sb, sh, ss)
    assert K.shape[2] + token0 >= chunk_end * cfg.chunk and chunk_begin * cfg.chunk >= token0
    assert expert.dtype == torch.uint8 and expert.dim() == 2 and expert.is_contiguous() and expert.is_cuda
    assert chunk_off.dtype == torch.int64 and chunk_off.dim() == 2 and chunk_off.is_contiguous()
    assert arena.dtype == torch.uint8 and arena.numel() >= pool_arena_bytes(cfg, n_pages) and status.dtype == torch.int32
    assert state.numel() * state.element_size() >= pool_state_bytes(cfg, n_pages)
    W = (None, None, None, None)
    if router is not None:
        W = router
        for w in W[:3]:
            assert w.is_cuda and w.dtype == torch.float16 and w.is_contiguous()
        if W[3] is not None:
            assert W[3].is_cuda and W[3].dtype == torch.float32
    if votes is not None:
        assert votes.dtype == torch.int32 and votes.is_contiguous() and votes.shape[:2] == expert.shape
    shift = token0 * ss * 2
    _check(lib().moqae_route_pack_paged(C.byref(cfg.c()), C.byref(_pc(n_pages)), C.c_void_p(K.data_ptr() - shift),
                                        C.c_void_p(V.data_ptr() - shift), sb, sh, ss, chunk_begin, chunk_end,
                                        _ptr(W[0]), _ptr(W[1]), _ptr(W[2]), _ptr(W[3]), _ptr(expert), expert.shape[1], _ptr(votes),
                                        _ptr(arena), _ptr(state), _ptr(chunk_off), chunk_off.shape[1], _ptr(status), _stream()),
           "moqae_route_pack_paged")


def pool_release(cfg: Cfg, n_pages: Sequence[int], expert: torch.Tensor, chunk_off: torch.Tensor, row_begin: int, row_end: int,
                 chunk_begin: int, chunk_end: int, state: torch.Tensor) -> None:
    assert expert.dtype == torch.uint8 and expert.is_contiguous() and chunk_off.dtype == torch.int64 and chunk_off.is_contiguous()
    _check(lib().moqae_pool_release(C.byref(cfg.c()), C.byref(_pc(n_pages)), _ptr(expert), expert.shape[1], _ptr(chunk_off),
                                    chunk_off.shape[1], row_begin, row_end, chunk_begin, chunk_end, _ptr(state), _stream()),
           "moqae_pool_release")


def decode_plan(cfg: Cfg, expert: Optional[torch.Tensor], n_chunks: int, workspace: torch.Tensor) -> None:
    """Leaves in `workspace` what decode_attn(..., planned=True) calls on these tables need."""
    stride = 0
    if n_chunks > 0:
        assert expert.dtype == torch.uint8 and expert.is_contiguous() and expert.is_cuda
        stride = expert.shape[1]
    _check(lib().moqae_decode_plan(C.byref(cfg.c()), _ptr(expert), stride, n_chunks, _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()), "moqae_decode_plan")


def decode_attn(cfg: Cfg, q: torch.Tensor, arena: Optional[torch.Tensor], chunk_off: Optional[torch.Tensor],
                expert: Optional[torch.Tensor], n_chunks: int,
                K_tail: Optional[torch.Tensor], V_tail: Optional[torch.Tensor], n_tail: int,
                softmax_scale: float, out: torch.Tensor, workspace: torch.Tensor, planned: bool = False) -> None:
    """q: fp16 [B, Hq, D]; out: fp32 [B, Hq, D]; workspace: uint8, >= decode_workspace_bytes().
    planned: the workspace holds a plan made by decode_plan for these tables (moqae_decode_attn_planned)."""
    assert q.is_cuda and q.dtype == torch.float16 and q.is_contiguous()
    assert q.shape == (cfg.batch, cfg.n_q_heads, cfg.head_dim)
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
    stride = 0
    if n_chunks > 0:
        assert expert.dtype == torch.uint8 and chunk_off.dtype == torch.int64
        assert expert.shape == chunk_off.shape and expert.is_contiguous() and chunk_off.is_contiguous()
        stride = expert.shape[1]
    if n_tail > 0:
        for t in (K_tail, V_tail):
            assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous()
            assert t.shape == (cfg.batch, cfg.n_kv_heads, cfg.chunk, cfg.head_dim)
    fn = lib().moqae_decode_attn_planned if planned else lib().moqae_decode_attn
    _check(fn(C.byref(cfg.c()), _ptr(q), _ptr(arena), _ptr(chunk_off), _ptr(expert), stride,
              n_chunks, _ptr(K_tail), _ptr(V_tail), n_tail, float(softmax_scale), _ptr(out),
              _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "moqae_decode_attn_planned" if planned else "moqae_decode_attn")


def decode_workspace_bytes_multi(cfg: Cfg, n_chunks: int, n_queries: int) -> int:
    return int(lib().moqae_decode_workspace_bytes_multi(C.byref(cfg.c()), n_chunks, n_queries))


def decode_attn_multi(cfg: Cfg, q: torch.Tensor, arena: Optional[torch.Tensor], chunk_off: Optional[torch.Tensor],
                      expert: Optional[torch.Tensor], n_chunks: int, K_tail: torch.Tensor, V_tail: torch.Tensor, n_tail: int,
                      softmax_scale: float, out: torch.Tensor, workspace: torch.Tensor) -> None:
    """q: fp16 [B, Q, Hq, D] (Q new tokens whose K, V rows are the last Q valid residual rows); out: fp32 [B, Q, Hq, D]."""
    assert q.is_cuda and q.dtype == torch.float16 and q.is_contiguous() and q.dim() == 4
    B, Q, Hq, D = q.shape
    assert (B, Hq, D) == (cfg.batch, cfg.n_q_heads, cfg.head_dim)
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
    stride = 0
    if n_chunks > 0:
        assert expert.dtype == torch.uint8 and chunk_off.dtype == torch.int64
        assert expert.shape == chunk_off.shape and expert.is_contiguous() and chunk_off.is_contiguous()
        stride = expert.shape[1]
    for t in (K_tail, V_tail):
        assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous()
        assert t.shape == (cfg.batch, cfg.n_kv_heads, cfg.chunk, cfg.head_dim)
    _check(lib().moqae_decode_attn_multi(C.byref(cfg.c()), _ptr(q), Q, _ptr(arena), _ptr(chunk_off), _ptr(expert), stride,
                                         n_chunks, _ptr(K_tail), _ptr(V_tail), n_tail, float(softmax_scale), _ptr(out),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "moqae_decode_attn_multi")


def static_scratch_bytes() -> int:
    return int(lib().moqae_static_scratch_bytes())


def decode_attn_static(cfg: Cfg, q: torch.Tensor, arena: Optional[torch.Tensor], chunk_off: Optional[torch.Tensor],
                       expert: Optional[torch.Tensor], n_chunks: int,
                       K_tail: Optional[torch.Tensor], V_tail: Optional[torch.Tensor], n_tail: int,
                       softmax_scale: float, out: torch.Tensor) -> None:
    """decode_attn on the library's own fixed scratch array (moqae_decode_attn_static): no workspace, no allocation."""
    assert q.is_cuda and q.dtype == torch.float16 and q.is_contiguous()
    assert q.shape == (cfg.batch, cfg.n_q_heads, cfg.head_dim)
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
    stride = 0
    if n_chunks > 0:
        assert expert.dtype == torch.uint8 and chunk_off.dtype == torch.int64
        assert expert.shape == chunk_off.shape and expert.is_contiguous() and chunk_off.is_contiguous()
        stride = expert.shape[1]
    if n_tail > 0:
        for t in (K_tail, V_tail):
            assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous()
            assert t.shape == (cfg.batch, cfg.n_kv_heads, cfg.chunk, cfg.head_dim)
    _check(lib().moqae_decode_attn_static(C.byref(cfg.c()), _ptr(q), _ptr(arena), _ptr(chunk_off), _ptr(expert), stride,
                                          n_chunks, _ptr(K_tail), _ptr(V_tail), n_tail, float(softmax_scale), _ptr(out),
                                          _stream()), "moqae_decode_attn_static")


def decode_attn_ragged(cfg: Cfg, q: torch.Tensor, arena: Optional[torch.Tensor], chunk_off: Optional[torch.Tensor],
                       expert: Optional[torch.Tensor], n_chunks_seq: torch.Tensor, max_chunks: int,
                       K_tail: torch.Tensor, V_tail: torch.Tensor, n_tail_seq: torch.Tensor,
                       softmax_scale: float, out: torch.Tensor, workspace: torch.Tensor) -> None:
    """As decode_attn with per-sequence lengths: n_chunks_seq, n_tail_seq int32 [B] on the GPU;
    workspace: uint8, >= decode_workspace_bytes_ragged(cfg, max_chunks)."""
    assert q.is_cuda and q.dtype == torch.float16 and q.is_contiguous()
    assert q.shape == (cfg.batch, cfg.n_q_heads, cfg.head_dim)
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
    for t in (n_chunks_seq, n_tail_seq):
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.shape == (cfg.batch,)
    stride = 0
    if max_chunks > 0:
        assert expert.dtype == torch.uint8 and chunk_off.dtype == torch.int64
        assert expert.shape == chunk_off.shape and expert.is_contiguous() and chunk_off.is_contiguous()
        stride = expert.shape[1]
    for t in (K_tail, V_tail):
        assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous()
        assert t.shape == (cfg.batch, cfg.n_kv_heads, cfg.chunk, cfg.head_dim)
    _check(lib().moqae_decode_attn_ragged(C.byref(cfg.c()), _ptr(q), _ptr(arena), _ptr(chunk_off), _ptr(expert), stride,
                                          _ptr(n_chunks_seq), max_chunks, _ptr(K_tail), _ptr(V_tail), _ptr(n_tail_seq),
                                          float(softmax_scale), _ptr(out), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream()),
           "moqae_decode_attn_ragged")


def append_tail(cfg: Cfg, k_new: torch.Tensor, v_new: torch.Tensor, K_tail: torch.Tensor, V_tail: torch.Tensor,
                n_tail: int) -> None:
    """k_new, v_new: fp16 [B, Hkv, D] -> row n_tail of K_tail, V_tail (fp16 [B, Hkv, N, D])."""
    for t in (k_new, v_new):
        assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous()
        assert t.shape == (cfg.batch, cfg.n_kv_heads, cfg.head_dim)
    for t in (K_tail, V_tail):
        assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous()
        assert t.shape == (cfg.batch, cfg.n_kv_heads, cfg.chunk, cfg.head_dim)
    _check(lib().moqae_append_tail(C.byref(cfg.c()), _ptr(k_new), _ptr(v_new), _ptr(K_tail), _ptr(V_tail), n_tail,
                                   _stream()), "moqae_append_tail")
