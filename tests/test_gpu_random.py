"""Seeded randomized parity: 320 random shapes through the C ABI against the CPU oracle, stopping at the first
failure.  A quarter each: uniform decode attention (<= 2e-3), ragged decode attention (<= 2e-3), quantise-and-pack
on scaled data (arena bytes and offsets bit-exact), the fused route + pack call on the paged store (decisions, votes,
placement and page bytes).  Bounded to well under a minute on the GPU."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import test_gpu_parity as T                                              # noqa: E402  (helpers only)
import test_gpu_paged as P                                               # noqa: E402  (helpers only)

mq = T.mq                                                                # the module-scoped binding fixture
N_CASES = 320


def test_random_shapes(mq, ref):
    rng = np.random.default_rng(12345)
    worst = 0.0
    for n in range(N_CASES):
        kind = n % 4
        N = int(rng.choice([8, 16, 32, 64, 128, 192, 256])); G = int(rng.choice([32, 64]))
        Hkv = int(rng.choice([1, 2, 3, 4])); rep = int(rng.choice([1, 1, 2, 4] if G == 64 else [1, 1, 2]))
        Hq = Hkv * rep; B = int(rng.choice([1, 2, 3]))
        seed = int(rng.integers(1 << 30))
        what = (n, kind, B, Hq, Hkv, N, G, seed)
        print(f"[random-case] {what}", file=sys.stderr, flush=True)
        if kind == 0:
            C = int(rng.integers(0, 40)); Tt = int(rng.integers(0, N))
            if C + Tt == 0:
                Tt = 1
            err = T._attn_case(mq, ref, B, Hq, Hkv, N, G, C, Tt, (2, 4, 8, 16), seed)
        elif kind == 1:
            lens = [int(rng.integers(0, 30 * N)) for _ in range(int(rng.integers(1, 5)))]
            err = T._ragged_case(mq, ref, Hq, Hkv, N, G, lens, seed=seed)
        elif kind == 3:
            r2 = np.random.default_rng(seed)
            C = int(r2.integers(1, 10)); freeze = int(r2.integers(0, 2))
            cfg, rcfg = T._cfgs(mq, ref, B, Hkv, Hkv, N, G, P.BITS, freeze)
            K, V = T._rand_kv(r2, B, Hkv, C * N)
            K *= np.float16(r2.choice([1e-2, 1.0, 30.0])); V *= np.float16(r2.choice([1e-3, 1.0, 50.0]))
            W = [(r2.standard_normal(sh) * 0.3).astype(np.float16) for sh in ((128, 4), (128, 4), (4, 4))]
            e_ref, v_ref = ref.route_chunks(rcfg, K, 0, C, *W)
            pages = tuple(int((e_ref == j).sum()) + 2 for j in range(4))
            arena = torch.zeros(mq.pool_arena_bytes(cfg, pages), dtype=torch.uint8, device="cuda")
            state = torch.zeros(mq.pool_state_bytes(cfg, pages) // 4, dtype=torch.int32, device="cuda")
            mq.pool_init(cfg, pages, state)
            expert = torch.full((B * Hkv, C), 255, dtype=torch.uint8, device="cuda")
            votes = torch.full((B * Hkv, C, 4), -1, dtype=torch.int32, device="cuda")
            off = torch.zeros((B * Hkv, C), dtype=torch.int64, device="cuda"); status = torch.zeros(1, dtype=torch.int32, device="cuda")
            mq.route_pack_paged(cfg, pages, T._dev(K), T._dev(V), 0, C, tuple(T._dev(w) for w in W) + (None,), expert, votes, arena, state, off, status)
            torch.cuda.synchronize()
            assert int(status.item()) == 0, what
            assert np.array_equal(expert.cpu().numpy(), e_ref) and np.array_equal(votes.cpu().numpy(), v_ref), what
            P._check_pages(mq, ref, cfg, rcfg, pages, K, V, e_ref, off.cpu().numpy().astype(np.uint64), arena.cpu().numpy(), 0, C)
            assert mq.pool_free_pages(cfg, pages, state) == [2, 2, 2, 2], what
            err = 0.0
        else:
            r2 = np.random.default_rng(seed)
            C = int(r2.integers(1, 12))
            cfg, rcfg = T._cfgs(mq, ref, B, Hkv, Hkv, N, G, (2, 4, 8, 16), 1)
            K, V = T._rand_kv(r2, B, Hkv, C * N)
            K *= np.float16(r2.choice([1e-4, 1.0, 300.0])); V *= np.float16(r2.choice([1e-3, 1.0, 50.0]))
            expert = r2.integers(0, 4, (B * Hkv, C)).astype(np.uint8)
            (arena, used, off, status), (arena_ref, used_ref, off_ref, st_ref) = T._pack_both(mq, ref, cfg, rcfg, K, V, 0, C, expert)
            assert int(status.item()) == 0 and int(used.item()) == int(used_ref[0]), what
            assert np.array_equal(off.cpu().numpy().astype(np.uint64), off_ref), what
            assert np.array_equal(arena.cpu().numpy(), arena_ref), what
            err = 0.0
        assert err <= T.ATTN_TOL, (what, err)
        worst = max(worst, err)
    print(f"[random] {N_CASES} cases, worst attention error {worst:.2e}", file=sys.stderr, flush=True)
