"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its host helpers agree with the closed forms."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mq():
    from paper_2506_07533_amd import binding
    if not os.path.exists(binding._LIB_PATH):
        from paper_2506_07533_amd import build
        build.build_lib()
    binding.lib()
    return binding


def test_every_declared_symbol_is_exported(mq):
    for fname, exports in (("moqae.h", mq.EXPORTS), ("moqae_bench.h", mq.BENCH_EXPORTS)):
        header = open(os.path.join(ROOT, "include", fname)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared = sorted(set(re.findall(r"\b(moqae_[a-z_0-9]+)\s*\(", header)))
        assert declared == sorted(exports), fname
        for name in declared:
            assert getattr(mq.lib(), name) is not None
    assert mq.abi_version() == 2
    assert "arena" in mq.strerror(mq.E_ARENA) and mq.strerror(0) == "ok"


def test_block_sizes_closed_form(mq):
    cfg = mq.Cfg(1, 40, 40, 128, 128, 64, (2, 4, 8, 16), 1)
    assert [mq.chunk_block_bytes(cfg, b) for b in (2, 4, 8, 16)] == [10240, 18432, 34816, 65536]
    cfg1 = mq.Cfg(1, 8, 8, 128, 64, 32, (2, 4, 8, 16), 1)
    assert [mq.chunk_block_bytes(cfg1, b) for b in (2, 4, 8, 16)] == [6144, 10240, 18432, 32768]
    cfg4 = mq.Cfg(4, 32, 8, 128, 256, 64, (2, 4, 8, 16), 1)
    assert [mq.chunk_block_bytes(cfg4, b) for b in (2, 4, 8, 16)] == [20480, 36864, 69632, 131072]
    assert mq.chunk_block_bytes(cfg, 3) == 0
    assert mq.arena_upper_bound(cfg, 10) == 256 + 10 * 65536
    ws = mq.decode_workspace_bytes(cfg, 1024)
    # 40 ticket counters 256 bytes apart and two words per row (unit count, workgroup count), rounded up to
    # 256 bytes; then whole partials (o[128], m, l) for each of the 40 query heads
    head = (40 * 256 + 2 * 40 * 4 + 255) // 256 * 256
    assert ws > head and (ws - head) % (40 * 130 * 4) == 0


@pytest.mark.parametrize("kw", [dict(head_dim=64), dict(group=16), dict(chunk=48), dict(chunk=512),
                                dict(n_q_heads=24), dict(expert_bits=(2, 3)), dict(expert_bits=()),
                                dict(n_q_heads=48, n_kv_heads=16), dict(freeze_chunks=-1), dict(batch=0)])
def test_invalid_configurations_are_rejected(mq, kw):
    base = dict(batch=1, n_q_heads=8, n_kv_heads=8, head_dim=128, chunk=128, group=64,
                expert_bits=(2, 4, 8, 16), freeze_chunks=1)
    base.update(kw)
    assert mq.chunk_block_bytes(mq.Cfg(**base), 2) == 0


def test_null_pointers_are_rejected_before_any_launch(mq):
    """Argument errors are found on the host, so this is safe without a GPU."""
    import ctypes as C
    cfg = mq.Cfg(1, 8, 8).c()
    L = mq.lib()
    assert L.moqae_route_chunks(C.byref(cfg), None, 0, 0, 128, 0, 1, None, None, None, None, None, 1, None, None) == mq.E_INVAL
    assert L.moqae_quantize_pack(C.byref(cfg), None, None, 0, 0, 128, 0, 1, None, 1, None, 0, None, None, 1, None, None) == mq.E_INVAL
    assert L.moqae_decode_attn(C.byref(cfg), None, None, None, None, 0, 0, None, None, 0, 1.0, None, None, 0, None) == mq.E_INVAL
    assert L.moqae_decode_attn_ragged(C.byref(cfg), None, None, None, None, 0, None, 4, None, None, None, 1.0, None, None, 0,
                                      None) == mq.E_INVAL
    assert mq.decode_workspace_bytes_ragged(mq.Cfg(1, 8, 8), 16) >= mq.decode_workspace_bytes(mq.Cfg(1, 8, 8), 16)
    assert L.moqae_append_tail(C.byref(cfg), None, None, None, None, 0, None) == mq.E_INVAL
    assert L.moqae_decode_plan(C.byref(cfg), None, 0, 4, None, 0, None) == mq.E_INVAL
    assert L.moqae_decode_attn_planned(C.byref(cfg), None, None, None, None, 0, 0, None, None, 0, 1.0, None, None, 0, None) == mq.E_INVAL


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; `bench.py --gpus N` with N > 1 says so and exits (before touching any GPU)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
