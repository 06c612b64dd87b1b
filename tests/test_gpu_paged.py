"""GPU parity of the paged store (moqae_route_pack_paged, moqae_pool_release) against the CPU oracle.

Which free page a chunk receives is not specified, so offsets are not compared; instead the check is complete on
what must hold: every chunk's page lies in the pool of its expert on a page boundary, no page is used twice, the
pool counters moved by the number of chunks, routing decisions and votes equal the oracle's, and the bytes of every
page equal the block the oracle packed for that chunk.  Decode attention then reads the paged store as any other."""
import math
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import test_gpu_parity as T                                              # noqa: E402  (helpers only)

mq = T.mq
BITS = (2, 4, 8, 16)
NONE = np.uint64(0xFFFFFFFFFFFFFFFF)


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", file=sys.stderr, flush=True)
    yield


def _check_pages(mq, ref, cfg, rcfg, pages, K, V, expert_h, off_h, arena_h, c0, c1):
    BH = expert_h.shape[0]
    N = cfg.chunk
    seen = set()
    for u in range(BH):
        b, h = divmod(u, cfg.n_kv_heads)
        for c in range(c0, c1):
            j = int(expert_h[u, c]); o = int(off_h[u, c]); pb = mq.pool_page_bytes(cfg, j)
            base = mq.pool_base(cfg, pages, j)
            assert base <= o < base + pages[j] * pb and (o - base) % pb == 0, (u, c, j, o)
            assert o not in seen, (u, c)
            seen.add(o)
            blk = ref.pack_chunk(rcfg, BITS[j], K[b, h, c * N:(c + 1) * N], V[b, h, c * N:(c + 1) * N])
            assert np.array_equal(arena_h[o:o + blk.size], blk), (u, c, j)
    return seen


@pytest.mark.parametrize("B,Hkv,N,G,C,freeze,kpc", [(1, 8, 64, 32, 12, 1, 0), (2, 3, 128, 64, 9, 1, 0), (1, 2, 256, 64, 5, 0, 0),
                                                   (2, 2, 32, 64, 21, 2, 0), (1, 3, 192, 32, 4, 1, 0),
                                                   (2, 2, 16, 64, 25, 1, 0), (1, 3, 8, 32, 30, 1, 0),       # small chunks
                                                   (1, 3, 128, 64, 7, 1, 1)])       # keys quantised per channel
def test_route_pack_paged(mq, ref, B, Hkv, N, G, C, freeze, kpc):
    rng = np.random.default_rng(B * 100 + N + C)
    cfg, rcfg = T._cfgs(mq, ref, B, Hkv, Hkv, N, G, BITS, freeze, kpc)
    BH = B * Hkv
    K, V = T._rand_kv(rng, B, Hkv, C * N)
    W = [(rng.standard_normal(s) * 0.3).astype(np.float16) for s in ((128, 4), (128, 4), (4, 4))]
    bias = (rng.standard_normal(4) * 0.05).astype(np.float32)
    e_ref, v_ref = ref.route_chunks(rcfg, K, 0, C, *W, bias)
    pages = tuple(int((e_ref == j).sum()) + 3 for j in range(4))
    arena = torch.zeros(mq.pool_arena_bytes(cfg, pages), dtype=torch.uint8, device="cuda")
    state = torch.zeros(mq.pool_state_bytes(cfg, pages) // 4, dtype=torch.int32, device="cuda")
    mq.pool_init(cfg, pages, state)
    expert = torch.full((BH, C), 255, dtype=torch.uint8, device="cuda")
    votes = torch.full((BH, C, 4), -1, dtype=torch.int32, device="cuda")
    off = torch.zeros((BH, C), dtype=torch.int64, device="cuda"); status = torch.zeros(1, dtype=torch.int32, device="cuda")
    Kd, Vd = T._dev(K), T._dev(V)
    router = tuple(T._dev(w) for w in W) + (T._dev(bias),)
    # two calls: chunks [0, C-2), then the rest (as a decode loop appends them)
    mq.route_pack_paged(cfg, pages, Kd, Vd, 0, C - 2, router, expert, votes, arena, state, off, status)
    mq.route_pack_paged(cfg, pages, Kd, Vd, C - 2, C, router, expert, votes, arena, state, off, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert np.array_equal(expert.cpu().numpy(), e_ref) and np.array_equal(votes.cpu().numpy(), v_ref)
    off_h = off.cpu().numpy().astype(np.uint64); arena_h = arena.cpu().numpy()
    _check_pages(mq, ref, cfg, rcfg, pages, K, V, e_ref, off_h, arena_h, 0, C)
    assert mq.pool_free_pages(cfg, pages, state) == [3, 3, 3, 3]                                    # every pool was sized demand + 3
    # pool geometry equals the oracle's closed forms
    assert mq.pool_arena_bytes(cfg, pages) == ref.pool_arena_bytes(rcfg, pages)
    assert [mq.pool_base(cfg, pages, j) for j in range(4)] == [ref.pool_base(rcfg, pages, j) for j in range(4)]

    # decode attention over the paged store against the oracle's own paged store
    arena_r = np.zeros(ref.pool_arena_bytes(rcfg, pages), np.uint8); state_r = ref.pool_init(rcfg, pages)
    e_r2 = np.full((BH, C), 255, np.uint8); off_r = np.zeros((BH, C), np.uint64)
    assert ref.route_pack_paged(rcfg, pages, K, V, 0, C, (*W, bias), e_r2, None, arena_r, state_r, off_r) == 0
    q = rng.standard_normal((B, Hkv, 128), dtype=np.float32).astype(np.float16)
    scale = 1 / math.sqrt(128)
    o_ref = ref.decode_attn(rcfg, q, arena_r, off_r, e_r2, C, None, None, 0, scale)
    out = torch.zeros((B, Hkv, 128), dtype=torch.float32, device="cuda")
    ws = torch.zeros(mq.decode_workspace_bytes(cfg, C), dtype=torch.uint8, device="cuda")
    mq.decode_attn(cfg, T._dev(q), arena, off, expert, C, None, None, 0, scale, out, ws)
    torch.cuda.synchronize()
    o = out.cpu().numpy().astype(np.float64)
    assert (np.abs(o - o_ref).max(-1) / np.abs(o_ref).max(-1)).max() <= T.ATTN_TOL


def test_release_reuse_shared_decisions_and_exhaustion(mq, ref):
    rng = np.random.default_rng(9)
    B, Hkv, N, G, C = 2, 2, 64, 64, 8
    cfg, rcfg = T._cfgs(mq, ref, B, Hkv, Hkv, N, G, BITS, 0)
    BH = B * Hkv
    K, V = T._rand_kv(rng, B, Hkv, C * N)
    expert_h = rng.integers(0, 4, (BH, C)).astype(np.uint8)
    need = [int((expert_h == j).sum()) for j in range(4)]
    pages = tuple(need)                                                  # exactly enough
    arena = torch.zeros(mq.pool_arena_bytes(cfg, pages), dtype=torch.uint8, device="cuda")
    state = torch.zeros(mq.pool_state_bytes(cfg, pages) // 4, dtype=torch.int32, device="cuda")
    mq.pool_init(cfg, pages, state)
    expert = T._dev(expert_h)
    off = torch.zeros((BH, C), dtype=torch.int64, device="cuda"); status = torch.zeros(1, dtype=torch.int32, device="cuda")
    Kd, Vd = T._dev(K), T._dev(V)
    # decisions given (a routing-sharing follower): no router
    mq.route_pack_paged(cfg, pages, Kd, Vd, 0, C, None, expert, None, arena, state, off, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and torch.equal(expert, T._dev(expert_h))
    off_h = off.cpu().numpy().astype(np.uint64)
    used = _check_pages(mq, ref, cfg, rcfg, pages, K, V, expert_h, off_h, arena.cpu().numpy(), 0, C)
    assert len(used) == BH * C
    # every pool is empty now: one more chunk per row fails with the arena status, and the chunks get no page
    off2 = torch.zeros((BH, 1), dtype=torch.int64, device="cuda")
    mq.route_pack_paged(cfg, pages, Kd, Vd, 0, 1, None, expert[:, :1].contiguous(), None, arena, state, off2, status)
    torch.cuda.synchronize()
    assert int(status.item()) == mq.E_ARENA and (off2.cpu().numpy().astype(np.uint64) == NONE).all()
    assert mq.pool_free_pages(cfg, pages, state) == [0, 0, 0, 0]
    # sticky: nothing happens while the status is set
    off3 = torch.full((BH, 1), 5, dtype=torch.int64, device="cuda")
    mq.route_pack_paged(cfg, pages, Kd, Vd, 0, 1, None, expert[:, :1].contiguous(), None, arena, state, off3, status)
    torch.cuda.synchronize()
    assert (off3 == 5).all().item()
    status.zero_()
    # give back the first three chunks of rows 1..2 and pack other data into the freed pages
    mq.pool_release(cfg, pages, expert, off, 1, 3, 0, 3, state)
    torch.cuda.synchronize()
    off_h2 = off.cpu().numpy().astype(np.uint64)
    assert (off_h2[1:3, :3] == NONE).all() and np.array_equal(off_h2[[0, 3]], off_h[[0, 3]]) and np.array_equal(off_h2[1:3, 3:], off_h[1:3, 3:])
    freed = {int(o) for o in off_h[1:3, :3].ravel()}
    assert mq.pool_free_pages(cfg, pages, state) == [int((expert_h[1:3, :3] == j).sum()) for j in range(4)]
    K2, V2 = T._rand_kv(rng, B, Hkv, C * N)
    K2d, V2d = T._dev(K2), T._dev(V2)
    mq.route_pack_paged(cfg, pages, K2d, V2d, 0, 3, None, expert, None, arena, state, off, status)     # all rows ask; rows 0 and 3 find nothing
    torch.cuda.synchronize()
    got = off.cpu().numpy().astype(np.uint64)
    assert int(status.item()) == mq.E_ARENA
    served = got[:, :3] != NONE
    assert int(served.sum()) == len(freed) and {int(o) for o in got[:, :3][served]} == freed
    arena_h = arena.cpu().numpy()
    for u in range(BH):
        b, h = divmod(u, Hkv)
        for c in range(3):
            if served[u, c]:
                j = int(expert_h[u, c])
                assert mq.pool_base(cfg, pages, j) <= int(got[u, c]) < mq.pool_base(cfg, pages, j) + pages[j] * mq.pool_page_bytes(cfg, j)
                blk = ref.pack_chunk(rcfg, BITS[j], K2[b, h, c * N:(c + 1) * N], V2[b, h, c * N:(c + 1) * N])
                assert np.array_equal(arena_h[int(got[u, c]):int(got[u, c]) + blk.size], blk)
