"""GPU parity on the five benchmark workloads at their full sizes, in the launch configuration
bench.py times.  Workloads 1-4 are compared in full (routing and packed bytes bit-exact,
attention within 2e-3); the 32-layer stack is compared on sampled (layer, sequence) slices.
"""
import dataclasses
import math
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", file=sys.stderr, flush=True)
    yield


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2506_07533_amd import binding, cache, synth
    from oracle import moqae_ref
    binding.lib(); moqae_ref.lib()
    return binding, cache, synth, moqae_ref


def _rel_err(o, o_ref):
    return float((np.abs(o - o_ref).max(-1) / np.abs(o_ref).max(-1)).max())


def _full_parity(env, name, n_decode=1, check_mix=False):
    mq, cache, synth, R = env
    w = synth.WORKLOADS[name]
    d = synth.make_workload(w)
    C, T, BH, M = w.n_chunks, w.n_tail, w.batch * w.n_kv_heads, len(w.expert_bits)
    cfg = mq.Cfg(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.chunk, w.group, w.expert_bits, w.freeze_chunks)
    rcfg = R.RefCfg(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.chunk, w.group, w.expert_bits, w.freeze_chunks)
    # oracle first: routing, then the arena
    e_ref, v_ref = R.route_chunks(rcfg, d["K"], 0, C, d["W1"], d["W2"], d["W3"])
    sizes = np.array([R.chunk_block_bytes(rcfg, b) for b in w.expert_bits], np.uint64)[e_ref]
    cap = int(sizes.sum()) + 4096
    arena_ref = np.zeros(cap, np.uint8); used_ref = np.zeros(1, np.uint64); off_ref = np.zeros((BH, C), np.uint64)
    assert R.quantize_pack(rcfg, d["K"], d["V"], 0, C, e_ref, arena_ref, used_ref, off_ref) == 0
    if check_mix:                                     # the planted classes are recovered, mix within 3 points
        share = np.bincount(e_ref[:, w.freeze_chunks:].ravel(), minlength=M) / e_ref[:, w.freeze_chunks:].size
        assert np.abs(share - np.array(w.mix)).max() < 0.03, share

    lc = cache.LayerCache(cfg, C, arena_bytes=cap)
    K = torch.from_numpy(d["K"]).cuda(); V = torch.from_numpy(d["V"]).cuda()
    router = tuple(torch.from_numpy(d[k]).cuda() for k in ("W1", "W2", "W3")) + (None,)
    lc.compress_prefill(K, V, router=router)
    torch.cuda.synchronize()
    lc.check_status()
    assert np.array_equal(lc.votes.cpu().numpy()[:, :C], v_ref)      # the cache's tables have whole 16-byte rows: C columns in use
    assert np.array_equal(lc.expert.cpu().numpy()[:, :C], e_ref)
    assert int(lc.arena_used.item()) == int(used_ref[0])
    assert np.array_equal(lc.chunk_off.cpu().numpy()[:, :C].astype(np.uint64), off_ref)
    got = lc.arena.cpu().numpy()
    bad = np.nonzero(got != arena_ref)[0]
    assert bad.size == 0, f"{bad.size} packed bytes differ, first at {bad[:4]}"
    del got, K, V

    scale = 1.0 / math.sqrt(w.head_dim)
    Kt = lc.K_tail.cpu().numpy(); Vt = lc.V_tail.cpu().numpy()
    out = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    errs = []
    for step in range(n_decode):                      # decisions taken once, tables reused by every call
        q = synth.make_q(w.batch, w.n_q_heads, w.head_dim, 1000 * w.seed + step)
        lc.decode(torch.from_numpy(q).cuda(), out, scale)
        torch.cuda.synchronize()
        o_ref = R.decode_attn(rcfg, q, arena_ref, off_ref, e_ref, C, Kt, Vt, T, scale)
        errs.append(_rel_err(out.cpu().numpy().astype(np.float64), o_ref))
    assert max(errs) <= ATTN_TOL, errs
    return errs


def test_tiny(env):
    _full_parity(env, "tiny")


def test_llama7b_32k(env):
    _full_parity(env, "llama7b_32k")


def test_llama13b_128k(env):
    _full_parity(env, "llama13b_128k", check_mix=True)


def test_gqa8b_128k_tables_reused_over_decode_calls(env):
    _full_parity(env, "gqa8b_128k", n_decode=3, check_mix=True)


@pytest.mark.parametrize("name", ["llama13b_128k", "gqa8b_128k"])
def test_route_pack_paged_full_size(env, name):
    """The fused route + pack call at full size: decisions and votes of every chunk against the oracle, every chunk on a
    page of its own in its expert's pool, the bytes of sampled pages against the oracle's block of that chunk."""
    mq, cache, synth, R = env
    w = synth.WORKLOADS[name]
    d = synth.make_workload(w)
    C, BH, M = w.n_chunks, w.batch * w.n_kv_heads, len(w.expert_bits)
    cfg = mq.Cfg(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.chunk, w.group, w.expert_bits, w.freeze_chunks)
    rcfg = R.RefCfg(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.chunk, w.group, w.expert_bits, w.freeze_chunks)
    e_ref, v_ref = R.route_chunks(rcfg, d["K"], 0, C, d["W1"], d["W2"], d["W3"])
    pages = tuple(int((e_ref == j).sum()) + 5 for j in range(M))
    arena = torch.zeros(mq.pool_arena_bytes(cfg, pages), dtype=torch.uint8, device="cuda")
    state = torch.zeros(mq.pool_state_bytes(cfg, pages) // 4, dtype=torch.int32, device="cuda")
    mq.pool_init(cfg, pages, state)
    expert = torch.full((BH, C), 255, dtype=torch.uint8, device="cuda")
    votes = torch.full((BH, C, M), -1, dtype=torch.int32, device="cuda")
    off = torch.zeros((BH, C), dtype=torch.int64, device="cuda"); status = torch.zeros(1, dtype=torch.int32, device="cuda")
    K = torch.from_numpy(d["K"]).cuda(); V = torch.from_numpy(d["V"]).cuda()
    router = tuple(torch.from_numpy(d[k]).cuda() for k in ("W1", "W2", "W3")) + (None,)
    mq.route_pack_paged(cfg, pages, K, V, 0, C, router, expert, votes, arena, state, off, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert np.array_equal(expert.cpu().numpy(), e_ref) and np.array_equal(votes.cpu().numpy(), v_ref)
    assert mq.pool_free_pages(cfg, pages, state) == [5] * M
    off_h = off.cpu().numpy().astype(np.uint64)
    assert np.unique(off_h).size == BH * C                            # no page handed out twice
    for j in range(M):                                                # every chunk in its expert's pool, on a page boundary
        o = off_h[e_ref == j].astype(np.int64) - mq.pool_base(cfg, pages, j)
        pb = mq.pool_page_bytes(cfg, j)
        assert ((o >= 0) & (o < pages[j] * pb) & (o % pb == 0)).all(), j
    rng = np.random.default_rng(7)
    N = w.chunk
    picks = [(int(rng.integers(BH)), int(rng.integers(C))) for _ in range(48)] + [(0, 0), (BH - 1, C - 1)]
    for j in range(M):                                                # and at least two chunks of every bit-width
        us, cs = np.nonzero(e_ref == j)
        picks += [(int(us[i]), int(cs[i])) for i in rng.choice(us.size, min(2, us.size), replace=False)]
    for u, c in picks:
        b, h = divmod(u, w.n_kv_heads)
        blk = R.pack_chunk(rcfg, w.expert_bits[int(e_ref[u, c])], d["K"][b, h, c * N:(c + 1) * N], d["V"][b, h, c * N:(c + 1) * N])
        o = int(off_h[u, c])
        got = arena[o:o + blk.size].cpu().numpy()
        assert np.array_equal(got, blk), (u, c, int(e_ref[u, c]))


@pytest.mark.parametrize("extra_tokens,flush_step", [(0, None), (96, 32)])
def test_stack32_sampled(env, extra_tokens, flush_step):
    """32 layers, routing shared by groups of 4, 64 decode steps that append one token per step.
    With 96 extra prefill tokens the residual fills up at step 32 and is flushed in every layer.
    Checked on sampled (layer, sequence) slices: a leader and a follower layer, two sequences."""
    mq, cache, synth, R = env
    w = synth.WORKLOADS["stack32_32k"]
    S0 = w.seq + extra_tokens
    N, D, B, H = w.chunk, w.head_dim, w.batch, w.n_kv_heads
    C0 = S0 // N
    M = len(w.expert_bits)
    cfg = mq.Cfg(B, w.n_q_heads, H, D, N, w.group, w.expert_bits, w.freeze_chunks)
    blk = [mq.chunk_block_bytes(cfg, b) for b in w.expert_bits]
    mean_blk = sum(s * p for s, p in zip(blk, w.mix))
    arena_bytes = int(B * H * (C0 + 2) * mean_blk * 1.08)
    stack = cache.KVStack(cfg, w.n_layers, w.share_group, C0 + 1, arena_bytes=[arena_bytes] * w.n_layers)
    layers_chk, seqs_chk = [4, 6], [0, 11]                       # layer 4 leads the group of layer 6
    keep = {}
    routers = {}
    for l in range(w.n_layers):
        d = synth.make_layer_device(w, l, "cuda", seq=S0)
        routers[l] = (d["W1"], d["W2"], d["W3"], None)
        stack.compress_prefill(l, d["K"], d["V"], routers)
        if l in layers_chk:
            keep[l] = {b: (d["K"][b].cpu().numpy(), d["V"][b].cpu().numpy()) for b in seqs_chk}
        del d
    torch.cuda.synchronize()
    for lc in stack.layers:
        lc.check_status()
    # routing sharing: followers carry the leader's table; the realised mix is the planted one
    e4 = stack.layers[4].expert.cpu().numpy()
    assert np.array_equal(stack.layers[6].expert.cpu().numpy(), e4)
    share = np.bincount(e4[:, w.freeze_chunks:C0].ravel(), minlength=M) / e4[:, w.freeze_chunks:C0].size
    assert np.abs(share - np.array(w.mix)).max() < 0.03, share

    # ---- decode: 64 steps, one new token per step and layer
    scale = 1.0 / math.sqrt(D)
    g = torch.Generator(device="cuda"); g.manual_seed(99)
    out = torch.zeros((B, w.n_q_heads, D), dtype=torch.float32, device="cuda")
    new_rows = {l: [] for l in layers_chk}
    outs = {}
    check_steps = {0, 31, 32, 63}
    for step in range(w.decode_steps):
        for l in range(w.n_layers):
            kn = torch.randn((B, H, D), generator=g, device="cuda", dtype=torch.float16)
            vn = torch.randn((B, H, D), generator=g, device="cuda", dtype=torch.float16)
            q = torch.randn((B, w.n_q_heads, D), generator=g, device="cuda", dtype=torch.float16)
            flushed = stack.append(l, kn, vn, routers)
            assert flushed == (flush_step is not None and step + 1 == flush_step), (step, l)
            stack.layers[l].decode(q, out, scale)
            if l in layers_chk:
                new_rows[l].append((kn[seqs_chk].cpu().numpy(), vn[seqs_chk].cpu().numpy()))
                if step in check_steps:
                    outs[(l, step)] = (q[seqs_chk].cpu().numpy(), out[seqs_chk].cpu().numpy().astype(np.float64))
    torch.cuda.synchronize()
    for lc in stack.layers:
        lc.check_status()
    n_steps = w.decode_steps
    S_end = S0 + n_steps
    assert all(lc.n_chunks == S_end // N and lc.n_tail == S_end % N for lc in stack.layers)
    if flush_step is not None:
        assert stack.layers[0].n_chunks == C0 + 1

    # ---- oracle on the sampled slices
    for l in layers_chk:
        lc = stack.layers[l]
        e_gpu = lc.expert.cpu().numpy().reshape(B, H, -1)
        off_gpu = lc.chunk_off.cpu().numpy().reshape(B, H, -1)
        for bi, b in enumerate(seqs_chk):
            Kb, Vb = keep[l][b]
            Kfull = np.concatenate([Kb] + [r[0][bi][:, None, :] for r in new_rows[l]], axis=1)[None]   # [1,H,S_end,D]
            Vfull = np.concatenate([Vb] + [r[1][bi][:, None, :] for r in new_rows[l]], axis=1)[None]
            rcfg = R.RefCfg(1, w.n_q_heads, H, D, N, w.group, w.expert_bits, w.freeze_chunks)
            C_end = S_end // N
            if l % w.share_group == 0:                        # the leader's decisions are the router's
                d0 = synth.make_router(D, M, w.seed, directions=synth.planted_directions(M, D, w.seed))
                e_ref, _ = R.route_chunks(rcfg, Kfull, 0, C_end, *d0, want_votes=False)
                assert np.array_equal(e_gpu[b, :, :C_end], e_ref)
            e_use = np.ascontiguousarray(e_gpu[b, :, :C_end])
            sizes = np.array(blk, np.uint64)[e_use]
            arena_ref = np.zeros(int(sizes.sum()) + 4096, np.uint8); used = np.zeros(1, np.uint64)
            off_ref = np.zeros((H, C_end), np.uint64)
            assert R.quantize_pack(rcfg, Kfull, Vfull, 0, C_end, e_use, arena_ref, used, off_ref) == 0
            # packed blocks, chunk by chunk (the GPU arena interleaves all sequences)
            arena_gpu = lc.arena
            for h in range(H):
                for c in list(range(0, C_end, 37)) + [C_end - 1]:
                    nb = int(sizes[h, c])
                    got = arena_gpu[int(off_gpu[b, h, c]): int(off_gpu[b, h, c]) + nb].cpu().numpy()
                    ref = arena_ref[int(off_ref[h, c]): int(off_ref[h, c]) + nb]
                    assert np.array_equal(got, ref), (l, b, h, c)
            # attention at the sampled steps: cache state after `step + 1` appended tokens
            for step in sorted(check_steps):
                S_t = S0 + step + 1
                C_t, T_t = S_t // N, S_t % N
                Kt = np.zeros((1, H, N, D), np.float16); Vt = np.zeros_like(Kt)
                Kt[0, :, :T_t] = Kfull[0, :, C_t * N:S_t]; Vt[0, :, :T_t] = Vfull[0, :, C_t * N:S_t]
                qh, o_gpu = outs[(l, step)]
                o_ref = R.decode_attn(rcfg, qh[bi][None], arena_ref, off_ref, e_use, C_t, Kt, Vt, T_t, scale)
                assert _rel_err(o_gpu[bi][None], o_ref) <= ATTN_TOL, (l, b, step)
