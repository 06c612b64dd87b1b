"""ctypes front-end of the CPU oracle (``moqae_ref.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  It imports nothing from the
GPU package and the GPU package imports nothing from here.

All arrays are host numpy arrays; fp16 tensors are passed as ``np.float16`` (or
``np.uint16`` bit patterns) and are C-contiguous in their last dimension.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moqae_ref.c")
_LIB = os.path.join(_HERE, "libmoqae_ref.so")

# -ffp-contract=off and no fast-math: every written operation rounds once.
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("chunk", C.c_int32), ("group", C.c_int32),
                ("n_experts", C.c_int32), ("expert_bits", C.c_int32 * 8),
                ("freeze_chunks", C.c_int32), ("k_per_channel", C.c_int32)]


@dataclass
class RefCfg:
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


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build(force=False))
        _lib.moqae_ref_half_to_float.restype = C.c_float
        _lib.moqae_ref_half_to_float.argtypes = [C.c_uint16]
        _lib.moqae_ref_float_to_half.restype = C.c_uint16
        _lib.moqae_ref_float_to_half.argtypes = [C.c_float]
        _lib.moqae_ref_exp_p.restype = C.c_float
        _lib.moqae_ref_exp_p.argtypes = [C.c_float]
        _lib.moqae_ref_chunk_block_bytes.restype = C.c_uint64
        _lib.moqae_ref_chunk_block_bytes.argtypes = [C.POINTER(_Cfg), C.c_int32]
        _lib.moqae_ref_quantize_group.restype = None
        _lib.moqae_ref_quantize_group.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        _lib.moqae_ref_pack_chunk.restype = None
        _lib.moqae_ref_pack_chunk.argtypes = [C.POINTER(_Cfg), C.c_int, C.c_void_p, C.c_void_p,
                                              C.c_int64, C.c_void_p]
        _lib.moqae_ref_decode_chunk.restype = None
        _lib.moqae_ref_decode_chunk.argtypes = [C.POINTER(_Cfg), C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.moqae_route_chunks_ref.restype = C.c_int
        _lib.moqae_route_chunks_ref.argtypes = [C.POINTER(_Cfg), C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                                C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        _lib.moqae_quantize_pack_ref.restype = C.c_int
        _lib.moqae_quantize_pack_ref.argtypes = [C.POINTER(_Cfg), C.c_void_p, C.c_void_p,
                                                 C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int32,
                                                 C.c_void_p, C.c_int64, C.c_void_p, C.c_uint64, C.c_void_p,
                                                 C.c_void_p, C.c_int64, C.c_void_p]
        _lib.moqae_decode_attn_ref.restype = C.c_int
        _lib.moqae_decode_attn_ref.argtypes = [C.POINTER(_Cfg), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                               C.c_double, C.c_void_p]
        _lib.moqae_ref_num_threads.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _h(a: np.ndarray) -> np.ndarray:
    """fp16 array -> its uint16 bit patterns (no copy when possible)."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def num_threads() -> int:
    return int(lib().moqae_ref_num_threads())


def half_to_float(bits: int) -> float:
    return float(lib().moqae_ref_half_to_float(int(bits)))


def float_to_half(x: float) -> int:
    return int(lib().moqae_ref_float_to_half(C.c_float(x)))


def exp_p(x: float) -> float:
    return float(lib().moqae_ref_exp_p(C.c_float(x)))


def chunk_block_bytes(cfg: RefCfg, bits: int) -> int:
    return int(lib().moqae_ref_chunk_block_bytes(C.byref(cfg.c()), bits))


def quantize_group(x: np.ndarray, bits: int):
    """One quantisation group: fp16 values -> (codes uint8[G], meta word)."""
    x = np.ascontiguousarray(_h(x))
    codes = np.zeros(x.size, np.uint8)
    meta = np.zeros(1, np.uint32)
    lib().moqae_ref_quantize_group(_p(x), x.size, bits, _p(codes), _p(meta))
    return codes, int(meta[0])


def pack_chunk(cfg: RefCfg, bits: int, Kc: np.ndarray, Vc: np.ndarray) -> np.ndarray:
    """Kc, Vc: [N, D] fp16 rows of one chunk -> the chunk block bytes."""
    Kc = np.ascontiguousarray(_h(Kc)); Vc = np.ascontiguousarray(_h(Vc))
    assert Kc.shape == (cfg.chunk, cfg.head_dim) == Vc.shape
    assert bits == 16 or ((cfg.chunk % 64 == 0 or cfg.chunk in (8, 16, 32)) and cfg.head_dim % 64 == 0), "V layout needs N % 64 == 0 or N in (8, 16, 32), and D % 64 == 0"
    blk = np.zeros(chunk_block_bytes(cfg, bits), np.uint8)
    lib().moqae_ref_pack_chunk(C.byref(cfg.c()), bits, _p(Kc), _p(Vc), cfg.head_dim, _p(blk))
    return blk


def decode_chunk(cfg: RefCfg, bits: int, blk: np.ndarray):
    """Chunk block bytes -> (K^, V^) as float64 [N, D]."""
    blk = np.ascontiguousarray(blk, np.uint8)
    assert blk.size >= chunk_block_bytes(cfg, bits)
    assert bits == 16 or ((cfg.chunk % 64 == 0 or cfg.chunk in (8, 16, 32)) and cfg.head_dim % 64 == 0), "V layout needs N % 64 == 0 or N in (8, 16, 32), and D % 64 == 0"
    Kh = np.zeros((cfg.chunk, cfg.head_dim), np.float64)
    Vh = np.zeros_like(Kh)
    lib().moqae_ref_decode_chunk(C.byref(cfg.c()), bits, _p(blk), _p(Kh), _p(Vh))
    return Kh, Vh


def _kv_strides(K: np.ndarray, cfg: RefCfg):
    assert K.ndim == 4 and K.shape[0] == cfg.batch and K.shape[1] == cfg.n_kv_heads
    assert K.shape[3] == cfg.head_dim and K.strides[3] == 2
    return K.strides[0] // 2, K.strides[1] // 2, K.strides[2] // 2


def route_chunks(cfg: RefCfg, K: np.ndarray, chunk_begin: int, chunk_end: int,
                 W1: np.ndarray, W2: np.ndarray, W3: np.ndarray,
                 bias: Optional[np.ndarray] = None,
                 expert: Optional[np.ndarray] = None, votes: Optional[np.ndarray] = None,
                 want_votes: bool = True):
    """K: [B, Hkv, S, D] fp16.  Returns (expert uint8 [B*Hkv, Ccap], votes int32 [B*Hkv, Ccap, M])."""
    K = _h(K)
    sb, sh, ss = _kv_strides(K, cfg)
    assert K.shape[2] >= chunk_end * cfg.chunk
    M = len(cfg.expert_bits)
    W1 = np.ascontiguousarray(_h(W1)); W2 = np.ascontiguousarray(_h(W2)); W3 = np.ascontiguousarray(_h(W3))
    assert W1.shape == (cfg.head_dim, M) == W2.shape and W3.shape == (M, M)
    if bias is not None:
        bias = np.ascontiguousarray(bias, np.float32); assert bias.shape == (M,)
    BH = cfg.batch * cfg.n_kv_heads
    if expert is None:
        expert = np.full((BH, chunk_end), 255, np.uint8)
    if votes is None and want_votes:
        votes = np.full((BH, expert.shape[1], M), -1, np.int32)
    rc = lib().moqae_route_chunks_ref(C.byref(cfg.c()), _p(K), sb, sh, ss, chunk_begin, chunk_end,
                                      _p(W1), _p(W2), _p(W3), _p(bias), _p(expert), expert.shape[1], _p(votes))
    if rc != 0:
        raise ValueError(f"moqae_route_chunks_ref -> {rc}")
    return expert, votes


def quantize_pack(cfg: RefCfg, K: np.ndarray, V: np.ndarray, chunk_begin: int, chunk_end: int,
                  expert: np.ndarray, arena: np.ndarray, arena_used: np.ndarray,
                  chunk_off: np.ndarray, status: Optional[np.ndarray] = None):
    """Packs into `arena` (uint8) from arena_used[0]; fills chunk_off (uint64 [B*Hkv, Ccap])."""
    K = _h(K); V = _h(V)
    sb, sh, ss = _kv_strides(K, cfg)
    assert _kv_strides(V, cfg) == (sb, sh, ss)
    assert K.shape[2] >= chunk_end * cfg.chunk
    assert expert.dtype == np.uint8 and expert.ndim == 2 and expert.flags.c_contiguous
    assert chunk_off.dtype == np.uint64 and chunk_off.ndim == 2 and chunk_off.flags.c_contiguous
    assert arena.dtype == np.uint8 and arena_used.dtype == np.uint64
    if status is None:
        status = np.zeros(1, np.int32)
    rc = lib().moqae_quantize_pack_ref(C.byref(cfg.c()), _p(K), _p(V), sb, sh, ss, chunk_begin, chunk_end,
                                       _p(expert), expert.shape[1], _p(arena), arena.size, _p(arena_used),
                                       _p(chunk_off), chunk_off.shape[1], _p(status))
    if rc != 0:
        raise ValueError(f"moqae_quantize_pack_ref -> {rc}")
    return int(status[0])


class _PoolCfg(C.Structure):
    _fields_ = [("n_pages", C.c_int32 * 8)]


def _pc(n_pages: Sequence[int]) -> _PoolCfg:
    return _PoolCfg((C.c_int32 * 8)(*(list(n_pages) + [0] * (8 - len(n_pages)))))


def pool_page_bytes(cfg: RefCfg, j: int) -> int:
    lib().moqae_ref_pool_page_bytes.restype = C.c_uint64
    return int(lib().moqae_ref_pool_page_bytes(C.byref(cfg.c()), C.c_int32(j)))


def pool_base(cfg: RefCfg, n_pages: Sequence[int], j: int) -> int:
    lib().moqae_ref_pool_base.restype = C.c_uint64
    return int(lib().moqae_ref_pool_base(C.byref(cfg.c()), C.byref(_pc(n_pages)), C.c_int32(j)))


def pool_arena_bytes(cfg: RefCfg, n_pages: Sequence[int]) -> int:
    lib().moqae_ref_pool_arena_bytes.restype = C.c_uint64
    return int(lib().moqae_ref_pool_arena_bytes(C.byref(cfg.c()), C.byref(_pc(n_pages))))


def pool_init(cfg: RefCfg, n_pages: Sequence[int]) -> np.ndarray:
    """Returns the pool state (uint32 words: head[8], tail[8], free rings)."""
    lib().moqae_ref_pool_state_bytes.restype = C.c_uint64
    nb = int(lib().moqae_ref_pool_state_bytes(C.byref(cfg.c()), C.byref(_pc(n_pages))))
    state = np.zeros(nb // 4, np.uint32)
    rc = lib().moqae_pool_init_ref(C.byref(cfg.c()), C.byref(_pc(n_pages)), _p(state))
    if rc != 0:
        raise ValueError(f"moqae_pool_init_ref -> {rc}")
    return state


def route_pack_paged(cfg: RefCfg, n_pages: Sequence[int], K: np.ndarray, V: np.ndarray, chunk_begin: int, chunk_end: int,
                     router, expert: np.ndarray, votes: Optional[np.ndarray], arena: np.ndarray, state: np.ndarray,
                     chunk_off: np.ndarray, status: Optional[np.ndarray] = None) -> int:
    """router: (W1, W2, W3, bias or None) or None (then `expert` holds the decisions to use).  Returns the status."""
    K = _h(K); V = _h(V)
    sb, sh, ss = _kv_strides(K, cfg)
    assert _kv_strides(V, cfg) == (sb, sh, ss) and K.shape[2] >= chunk_end * cfg.chunk
    assert expert.dtype == np.uint8 and expert.ndim == 2 and expert.flags.c_contiguous
    assert chunk_off.dtype == np.uint64 and chunk_off.ndim == 2 and chunk_off.flags.c_contiguous
    assert arena.dtype == np.uint8 and state.dtype == np.uint32
    if votes is not None:
        assert votes.dtype == np.int32 and votes.flags.c_contiguous
    if status is None:
        status = np.zeros(1, np.int32)
    W = [None, None, None, None]
    if router is not None:
        W = [_h(router[0]), _h(router[1]), _h(router[2]), None if router[3] is None else np.ascontiguousarray(router[3], np.float32)]
    pp = lambda a: None if a is None else _p(a)
    rc = lib().moqae_route_pack_paged_ref(C.byref(cfg.c()), C.byref(_pc(n_pages)), _p(K), _p(V), C.c_int64(sb), C.c_int64(sh),
                                          C.c_int64(ss), C.c_int32(chunk_begin), C.c_int32(chunk_end), pp(W[0]), pp(W[1]), pp(W[2]),
                                          pp(W[3]), _p(expert), C.c_int64(expert.shape[1]), pp(votes), _p(arena), _p(state),
                                          _p(chunk_off), C.c_int64(chunk_off.shape[1]), _p(status))
    if rc != 0:
        raise ValueError(f"moqae_route_pack_paged_ref -> {rc}")
    return int(status[0])


def pool_release(cfg: RefCfg, n_pages: Sequence[int], expert: np.ndarray, chunk_off: np.ndarray, row_begin: int, row_end: int,
                 chunk_begin: int, chunk_end: int, state: np.ndarray) -> None:
    rc = lib().moqae_pool_release_ref(C.byref(cfg.c()), C.byref(_pc(n_pages)), _p(expert), C.c_int64(expert.shape[1]),
                                      _p(chunk_off), C.c_int64(chunk_off.shape[1]), C.c_int32(row_begin), C.c_int32(row_end),
                                      C.c_int32(chunk_begin), C.c_int32(chunk_end), _p(state))
    if rc != 0:
        raise ValueError(f"moqae_pool_release_ref -> {rc}")


def decode_attn_multi(cfg: RefCfg, q: np.ndarray, arena, chunk_off, expert, n_chunks: int, K_tail: np.ndarray, V_tail: np.ndarray,
                      n_tail: int, softmax_scale: float) -> np.ndarray:
    """q: [B, Q, Hq, D] fp16; the Q new tokens' rows are the last Q valid residual rows.  Returns float64 [B, Q, Hq, D]."""
    q = np.ascontiguousarray(_h(q))
    B, Q, Hq, D = q.shape
    assert (B, Hq, D) == (cfg.batch, cfg.n_q_heads, cfg.head_dim)
    K_tail = np.ascontiguousarray(_h(K_tail)); V_tail = np.ascontiguousarray(_h(V_tail))
    out = np.zeros((B, Q, Hq, D), np.float64)
    stride = 0 if expert is None else expert.shape[1]
    rc = lib().moqae_decode_attn_multi_ref(C.byref(cfg.c()), _p(q), C.c_int32(Q), _p(arena), _p(chunk_off), _p(expert),
                                           C.c_int64(stride), C.c_int32(n_chunks), _p(K_tail), _p(V_tail), C.c_int32(n_tail),
                                           C.c_double(softmax_scale), _p(out))
    if rc != 0:
        raise ValueError(f"moqae_decode_attn_multi_ref -> {rc}")
    return out


def router_loss_grad(cfg: RefCfg, K: np.ndarray, token_begin: int, token_end: int, W1, W2, W3, bias, nll: np.ndarray,
                     pen_model: np.ndarray, pen_mem: np.ndarray, lam: float):
    """Eq. (3)-(5) over tokens [token_begin, token_end) of every (b, h).  Returns (loss[3] = L, L_model, L_mem,
    dW1 [D, M], dW2 [D, M], dW3 [M, M], dbias [M]) in float64."""
    K = _h(K); W1 = _h(W1); W2 = _h(W2); W3 = _h(W3)
    sb, sh, ss = _kv_strides(K, cfg)
    M, D = len(cfg.expert_bits), cfg.head_dim
    nll = np.ascontiguousarray(nll, np.float32); pen_model = np.ascontiguousarray(pen_model, np.float32)
    pen_mem = np.ascontiguousarray(pen_mem, np.float32)
    assert nll.shape == (cfg.batch,) and pen_model.shape == (M,) and pen_mem.shape == (M,)
    b = None if bias is None else np.ascontiguousarray(bias, np.float32)
    loss = np.zeros(3); dW1 = np.zeros((D, M)); dW2 = np.zeros((D, M)); dW3 = np.zeros((M, M)); db = np.zeros(M)
    rc = lib().moqae_router_loss_grad_ref(C.byref(cfg.c()), _p(K), C.c_int64(sb), C.c_int64(sh), C.c_int64(ss),
                                          C.c_int32(token_begin), C.c_int32(token_end), _p(W1), _p(W2), _p(W3), _p(b),
                                          _p(nll), _p(pen_model), _p(pen_mem), C.c_double(lam),
                                          _p(loss), _p(dW1), _p(dW2), _p(dW3), _p(db))
    if rc != 0:
        raise ValueError(f"moqae_router_loss_grad_ref -> {rc}")
    return loss, dW1, dW2, dW3, db


def decode_attn(cfg: RefCfg, q: np.ndarray, arena: Optional[np.ndarray], chunk_off: Optional[np.ndarray],
                expert: Optional[np.ndarray], n_chunks: int,
                K_tail: Optional[np.ndarray], V_tail: Optional[np.ndarray], n_tail: int,
                softmax_scale: float) -> np.ndarray:
    """q: [B, Hq, D] fp16; tails: [B, Hkv, N, D] fp16.  Returns float64 [B, Hq, D]."""
    q = np.ascontiguousarray(_h(q))
    assert q.shape == (cfg.batch, cfg.n_q_heads, cfg.head_dim)
    stride = 0
    if n_chunks > 0:
        assert expert.dtype == np.uint8 and chunk_off.dtype == np.uint64
        assert expert.shape == chunk_off.shape and expert.flags.c_contiguous and chunk_off.flags.c_contiguous
        stride = expert.shape[1]
    if n_tail > 0:
        K_tail = np.ascontiguousarray(_h(K_tail)); V_tail = np.ascontiguousarray(_h(V_tail))
        assert K_tail.shape == (cfg.batch, cfg.n_kv_heads, cfg.chunk, cfg.head_dim) == V_tail.shape
    out = np.zeros((cfg.batch, cfg.n_q_heads, cfg.head_dim), np.float64)
    rc = lib().moqae_decode_attn_ref(C.byref(cfg.c()), _p(q), _p(arena), _p(chunk_off), _p(expert), stride,
                                     n_chunks, _p(K_tail) if n_tail else None, _p(V_tail) if n_tail else None,
                                     n_tail, float(softmax_scale), _p(out))
    if rc != 0:
        raise ValueError(f"moqae_decode_attn_ref -> {rc}")
    return out
