"""Pins of the oracle's paged store (pools of fixed pages, one per expert) to things other than itself.

The store keeps the same chunk blocks as the ordered arena (whose packer is pinned by hand-worked words in
test_oracle_pins.py); what is new is the allocator, pinned here by closed forms and by a model of free rings
written out below with plain Python lists."""
import numpy as np
import pytest

BITS = (2, 4, 8, 16)


def _setup(ref, B=2, Hkv=2, N=64, G=64, C=6, seed=0):
    rng = np.random.default_rng(seed)
    cfg = ref.RefCfg(B, Hkv, Hkv, 128, N, G, BITS, 0)
    K = rng.standard_normal((B, Hkv, C * N, 128), dtype=np.float32).astype(np.float16)
    V = rng.standard_normal((B, Hkv, C * N, 128), dtype=np.float32).astype(np.float16)
    expert = rng.integers(0, 4, (B * Hkv, C)).astype(np.uint8)
    return cfg, K, V, expert


def test_pool_geometry_closed_form(ref):
    cfg = ref.RefCfg(1, 1, 1, 128, 128, 64, BITS, 0)
    pages = (5, 3, 2, 7)
    assert [ref.pool_page_bytes(cfg, j) for j in range(4)] == [10240, 18432, 34816, 65536]
    assert [ref.pool_base(cfg, pages, j) for j in range(4)] == [0, 51200, 51200 + 55296, 51200 + 55296 + 69632]
    assert ref.pool_arena_bytes(cfg, pages) == 51200 + 55296 + 69632 + 7 * 65536
    st = ref.pool_init(cfg, pages)
    assert st.size == 32 + sum(pages)
    assert list(st[:8]) == [0] * 8 and list(st[8:16]) == [5, 3, 2, 7, 0, 0, 0, 0]
    assert list(st[32:]) == [0, 1, 2, 3, 4, 0, 1, 2, 0, 1, 0, 1, 2, 3, 4, 5, 6]


def test_pages_follow_the_ring_model_and_hold_the_chunk_blocks(ref):
    """Allocation in (b, h, c) order takes ring[head] of the routed expert's pool; a released page goes to
    ring[tail] and is handed out again after the pages that were free before it (first in, first out)."""
    cfg, K, V, expert = _setup(ref)
    BH, C = expert.shape
    N = cfg.chunk
    pages = tuple(int((expert == j).sum()) + 2 for j in range(4))
    arena = np.zeros(ref.pool_arena_bytes(cfg, pages), np.uint8)
    state = ref.pool_init(cfg, pages)
    off = np.zeros((BH, C), np.uint64)
    # the model: one FIFO list of free pages per pool
    free = [list(range(n)) for n in pages]
    want = np.zeros((BH, C), np.uint64)

    def model_alloc(c0, c1):
        for u in range(BH):
            for c in range(c0, c1):
                j = int(expert[u, c])
                want[u, c] = ref.pool_base(cfg, pages, j) + free[j].pop(0) * ref.pool_page_bytes(cfg, j)

    assert ref.route_pack_paged(cfg, pages, K, V, 0, 4, None, expert, None, arena, state, off) == 0
    model_alloc(0, 4)
    assert np.array_equal(off[:, :4], want[:, :4])
    # every page holds the block the chunk packer makes for its chunk; no page twice; inside its pool
    seen = set()
    for u in range(BH):
        for c in range(4):
            j = int(expert[u, c]); o = int(off[u, c]); pb = ref.pool_page_bytes(cfg, j)
            assert (o - ref.pool_base(cfg, pages, j)) % pb == 0 and o not in seen
            assert ref.pool_base(cfg, pages, j) <= o < ref.pool_base(cfg, pages, j) + pages[j] * pb
            seen.add(o)
            b, h = divmod(u, cfg.n_kv_heads)
            blk = ref.pack_chunk(cfg, BITS[j], K[b, h, c * N:(c + 1) * N], V[b, h, c * N:(c + 1) * N])
            assert np.array_equal(arena[o:o + blk.size], blk)
    assert [int(state[j]) for j in range(4)] == [int((expert[:, :4] == j).sum()) for j in range(4)]
    # give back chunks 1..2 of rows 1..2, then allocate the rest: the released pages come after the never-used ones
    ref.pool_release(cfg, pages, expert, off, 1, 3, 1, 3, state)
    for u in range(1, 3):
        for c in range(1, 3):
            j = int(expert[u, c])
            free[j].append(int((want[u, c] - ref.pool_base(cfg, pages, j)) // ref.pool_page_bytes(cfg, j)))
            want[u, c] = np.uint64(0xFFFFFFFFFFFFFFFF)
    assert np.array_equal(off[:, :4], want[:, :4])
    assert ref.route_pack_paged(cfg, pages, K, V, 4, 6, None, expert, None, arena, state, off) == 0
    model_alloc(4, 6)
    assert np.array_equal(off, want)
    live = [int(o) for o in off.ravel() if o != np.uint64(0xFFFFFFFFFFFFFFFF)]
    assert len(live) == len(set(live)) == BH * C - 4


def test_routing_inside_the_paged_call_equals_route_chunks(ref):
    cfg, K, V, _ = _setup(ref, seed=3)
    rng = np.random.default_rng(5)
    W = [(rng.standard_normal(s) * 0.3).astype(np.float16) for s in ((128, 4), (128, 4), (4, 4))]
    BH, C = cfg.batch * cfg.n_kv_heads, 6
    e_want, v_want = ref.route_chunks(cfg, K, 0, C, *W)
    pages = (BH * C,) * 4
    arena = np.zeros(ref.pool_arena_bytes(cfg, pages), np.uint8)
    state = ref.pool_init(cfg, pages)
    expert = np.full((BH, C), 255, np.uint8); votes = np.zeros((BH, C, 4), np.int32); off = np.zeros((BH, C), np.uint64)
    assert ref.route_pack_paged(cfg, pages, K, V, 0, C, (*W, None), expert, votes, arena, state, off) == 0
    assert np.array_equal(expert, e_want) and np.array_equal(votes, v_want)


def test_an_empty_pool_sets_the_status_and_skips_the_chunk(ref):
    cfg, K, V, expert = _setup(ref, seed=7)
    BH, C = expert.shape
    need = [int((expert == j).sum()) for j in range(4)]
    pages = (need[0], need[1] - 2, need[2], need[3])                    # pool 1 is two pages short
    arena = np.zeros(ref.pool_arena_bytes(cfg, pages), np.uint8)
    state = ref.pool_init(cfg, pages)
    off = np.zeros((BH, C), np.uint64); status = np.zeros(1, np.int32)
    assert ref.route_pack_paged(cfg, pages, K, V, 0, C, None, expert, None, arena, state, off, status) == -3
    missing = off == np.uint64(0xFFFFFFFFFFFFFFFF)
    assert int(missing.sum()) == 2 and (expert[missing] == 1).all()
    # sticky: a further call does nothing
    before = state.copy()
    assert ref.route_pack_paged(cfg, pages, K, V, 0, C, None, expert, None, arena, state, off, status) == -3
    assert np.array_equal(state, before)
