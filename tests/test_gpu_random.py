"""Seeded randomized parity: 240 random shapes through the C ABI against the CPU oracle, stopping at the first
failure.  A third each: uniform decode attention (<= 2e-3), ragged decode attention (<= 2e-3), quantise-and-pack
on scaled data (arena bytes and offsets bit-exact).  Bounded to well under a minute on the GPU."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import test_gpu_parity as T                                              # noqa: E402  (helpers only)

mq = T.mq                                                                # the module-scoped binding fixture
N_CASES = 240


def test_random_shapes(mq, ref):
    rng = np.random.default_rng(12345)
    worst = 0.0
    for n in range(N_CASES):
        kind = n % 3
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
