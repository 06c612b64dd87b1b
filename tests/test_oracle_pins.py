"""Pins of the CPU oracle to things other than itself (no GPU needed).

Each test names the mistake it is meant to catch.  References: router Eq. (1)-(2)
and the residual rule of Sec. 3.2, routing freezing of Sec. 3.4, decode attention
of the "Limitations" section; the quantiser and the packed layout are this
build's own definition (the paper gives neither).
"""
import math
import os
import re

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# fp16 conversions and exp_p
# ----------------------------------------------------------------------------

def test_half_to_float_exhaustive(ref):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([ref.half_to_float(int(b)) for b in bits], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_float_to_half_rne(ref):
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * 3,
        (rng.standard_normal(5000) * 1e-6).astype(np.float32),          # subnormal halves
        np.float32(65504) * rng.uniform(0.9, 1.1, 2000).astype(np.float32),
        # exact half-way points between neighbouring halves (ties-to-even)
        ((np.arange(1, 4000, dtype=np.float64) + 0.5) * 2.0 ** -14).astype(np.float32),
        np.array([0.0, -0.0, 2.0 ** -25, 2.0 ** -24, 3 * 2.0 ** -25, 65519.99, 65520.0, 1e9, -1e9], np.float32),
    ])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([ref.float_to_half(float(x)) for x in xs], np.uint16)
    assert np.array_equal(got, want)


def test_exp_p_against_libm(ref):
    xs = np.concatenate([np.linspace(-80, 80, 4001), np.random.default_rng(2).uniform(-5, 5, 2000)])
    for x in xs:
        x32 = float(np.float32(x))
        assert abs(ref.exp_p(x32) / math.exp(x32) - 1.0) < 1e-5
    assert ref.exp_p(0.0) == 1.0
    assert ref.exp_p(-1000.0) == ref.exp_p(-80.0)                        # clamped
    assert ref.exp_p(1000.0) == ref.exp_p(80.0)


def test_exp_p_coefficients_are_taylor():
    """The constants written in the oracle are (ln 2)^k / k! rounded to binary32."""
    src = open(os.path.join(os.path.dirname(GOLD), "..", "oracle", "moqae_ref.c")).read()
    consts = {n: float.fromhex(v) for n, v in re.findall(r"\b(C[1-6]|LOG2E) = (0x[0-9a-fA-F.]+p[+-]?\d+)f", src)}
    assert sorted(consts) == ["C1", "C2", "C3", "C4", "C5", "C6", "LOG2E"]
    ln2 = math.log(2.0)
    for k in range(1, 7):
        assert np.float32(consts[f"C{k}"]) == np.float32(ln2 ** k / math.factorial(k)), k
    assert np.float32(consts["LOG2E"]) == np.float32(1.0 / ln2)


# ----------------------------------------------------------------------------
# Router: Eq. (1) and (2)
# ----------------------------------------------------------------------------

def _brute_router(K, W1, W2, W3, bias=None):
    """Eq. (1)-(2) in binary64 with library matmul: votes [C, M], margins [C, N]."""
    x = K.astype(np.float64)                                             # [C, N, D]
    z = (x @ W1.astype(np.float64)) * (x @ W2.astype(np.float64))
    h = z / (1.0 + np.exp(-z))
    p = h @ W3.astype(np.float64)
    if bias is not None:
        p = p + bias
    top = p.argmax(-1)
    srt = np.sort(p, -1)
    margin = srt[..., -1] - srt[..., -2]
    M = W3.shape[0]
    votes = np.stack([(top == k).sum(-1) for k in range(M)], -1)
    return votes, margin


@pytest.mark.parametrize("N,D,M", [(32, 8, 3), (64, 16, 4), (32, 128, 4), (96, 64, 5), (16, 128, 4), (8, 128, 4)])
def test_router_brute_force(ref, N, D, M):
    """A dropped term, SiLU on the wrong operand, a transposed W3 or a wrong
    vote rule all change the counts."""
    ok_seeds = 0
    for seed in range(6):
        rng = np.random.default_rng(seed)
        C = 5
        K = rng.standard_normal((1, 1, C * N, D)).astype(np.float16)
        W1 = (rng.standard_normal((D, M)) * 0.4).astype(np.float16)
        W2 = (rng.standard_normal((D, M)) * 0.4).astype(np.float16)
        W3 = (rng.standard_normal((M, M)) * 0.7).astype(np.float16)
        bias = rng.standard_normal(M).astype(np.float32) * 0.1 if seed % 2 else None
        bits = ([2, 4, 8, 16, 4, 8])[:M]
        cfg = ref.RefCfg(1, 1, 1, D, N, min(D, 32), bits, 0)
        expert, votes = ref.route_chunks(cfg, K, 0, C, W1, W2, W3, bias)
        bv, margin = _brute_router(K.reshape(C, N, D), W1, W2, W3, bias)
        assert votes.shape == (1, C, M) and (votes.sum(-1) == N).all()
        unsure = (margin < 1e-4).sum(-1)                                 # tokens whose top-1 fp32 may flip
        diff = np.abs(votes[0] - bv).sum(-1)
        assert (diff <= 2 * unsure).all()
        if unsure.sum() == 0:
            ok_seeds += 1
            assert np.array_equal(votes[0], bv)
            assert np.array_equal(expert[0], bv.argmax(-1))              # numpy argmax = first maximum
    assert ok_seeds >= 3


def test_router_one_hot_special_case(ref):
    """W1 = W2 = one-hot columns, W3 = permutation: logits[k] = SiLU(x[ch[perm^-1 k]]^2),
    so the token expert is decided by the largest |x| among the tapped channels."""
    rng = np.random.default_rng(7)
    N, D, M, C = 32, 64, 4, 6
    K = rng.standard_normal((2, 3, C * N, D)).astype(np.float16)
    ch = np.array([5, 17, 40, 63])
    perm = np.array([2, 0, 3, 1])                                        # hidden j feeds logit perm[j]
    W1 = np.zeros((D, M), np.float16); W1[ch, np.arange(M)] = 1
    W3 = np.zeros((M, M), np.float16); W3[np.arange(M), perm] = 1
    cfg = ref.RefCfg(2, 3, 3, D, N, 32, (2, 4, 8, 16), 0)
    expert, votes = ref.route_chunks(cfg, K, 0, C, W1, W1, W3)
    tapped = np.abs(K.astype(np.float64))[..., ch]                       # [2,3,S,M]
    tok = perm[tapped.argmax(-1)].reshape(6, C, N)
    want = np.stack([(tok == k).sum(-1) for k in range(M)], -1)
    assert np.array_equal(votes, want)


def test_router_vote_invariants_and_rf(ref):
    rng = np.random.default_rng(3)
    N, D, M, C = 64, 128, 4, 4
    K = rng.standard_normal((1, 2, C * N, D)).astype(np.float16)
    W = [(rng.standard_normal(s) * 0.3).astype(np.float16) for s in [(D, M), (D, M), (M, M)]]
    cfg = ref.RefCfg(1, 2, 2, D, N, 64, (2, 4, 16, 8), 2)
    e, v = ref.route_chunks(cfg, K, 0, C, *W)
    # routing freezing (Sec. 3.4): frozen chunks are the FP16 expert (index 2 here), not routed
    assert (e[:, :2] == 2).all() and (v[:, :2] == 0).all()
    assert (v[:, 2:].sum(-1) == N).all()
    # the vote does not depend on the order of the tokens inside a chunk
    Kp = K.reshape(1, 2, C, N, D)[:, :, :, rng.permutation(N)].reshape(K.shape)
    e2, v2 = ref.route_chunks(cfg, np.ascontiguousarray(Kp), 0, C, *W)
    assert np.array_equal(v, v2) and np.array_equal(e, e2)
    # a sub-range call writes only its own entries
    e3 = np.full_like(e, 255)
    ref.route_chunks(cfg, K, 3, 4, *W, expert=e3, want_votes=False)
    assert (e3[:, :3] == 255).all() and np.array_equal(e3[:, 3], e[:, 3])
    # no FP16 expert + freezing -> rejected
    W3e = [(rng.standard_normal(s) * 0.3).astype(np.float16) for s in [(D, 3), (D, 3), (3, 3)]]
    with pytest.raises(ValueError):
        ref.route_chunks(ref.RefCfg(1, 2, 2, D, N, 64, (2, 4, 8), 1), K, 0, C, *W3e)
    ref.route_chunks(ref.RefCfg(1, 2, 2, D, N, 64, (2, 4, 8), 0), K, 0, C, *W3e)


def test_router_ties_first_index_wins(ref):
    """All-zero weights give equal logits: token top-1 = expert 0; a bias that
    favours expert 2 on all tokens moves every vote there; an exact 50/50 vote
    between experts 1 and 3 resolves to the lower index."""
    N, D, M = 32, 16, 4
    K = np.random.default_rng(0).standard_normal((1, 1, N, D)).astype(np.float16)
    Z = np.zeros((D, M), np.float16); Z3 = np.zeros((M, M), np.float16)
    cfg = ref.RefCfg(1, 1, 1, D, N, 16, (2, 4, 8, 16), 0)
    e, v = ref.route_chunks(cfg, K, 0, 1, Z, Z, Z3)
    assert e[0, 0] == 0 and list(v[0, 0]) == [N, 0, 0, 0]
    e, v = ref.route_chunks(cfg, K, 0, 1, Z, Z, Z3, np.array([0, 0, 1, 1], np.float32))
    assert e[0, 0] == 2 and list(v[0, 0]) == [0, 0, N, 0]
    # half the rows light channel 0 (-> expert 1), half channel 1 (-> expert 3)
    K2 = np.zeros((1, 1, N, D), np.float16)
    K2[0, 0, ::2, 0] = 2.0
    K2[0, 0, 1::2, 1] = 2.0
    W1 = np.zeros((D, M), np.float16); W1[0, 1] = 1; W1[1, 3] = 1
    e, v = ref.route_chunks(cfg, K2, 0, 1, W1, W1, np.eye(M, dtype=np.float16))
    assert list(v[0, 0]) == [0, N // 2, 0, N // 2] and e[0, 0] == 1


# ----------------------------------------------------------------------------
# Quantiser and packing
# ----------------------------------------------------------------------------

def _read_groups():
    for line in open(os.path.join(GOLD, "quant_groups.txt")):
        if line.startswith("group"):
            bits, vals, meta, codes = [s.strip() for s in line[5:].split("|")]
            yield int(bits), [float(v) for v in vals.split()], int(meta, 16), [int(c) for c in codes.split()]


def test_quantize_group_golden(ref):
    n = 0
    for bits, vals, meta, codes in _read_groups():
        x = np.full(32, vals[0], np.float16)
        x[: len(vals)] = vals
        c, m = ref.quantize_group(x, bits)
        assert m == meta, (vals, hex(m))
        assert list(c[: len(vals)]) == codes
        assert (c[len(vals):] == codes[0]).all()
        n += 1
    assert n >= 8


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_quantize_group_invariants(ref, bits):
    """Codes in range, min -> 0, max -> qmax, |x - x^| <= scale/2, constant groups exact."""
    rng = np.random.default_rng(bits)
    qmax = (1 << bits) - 1
    for trial in range(400):
        G = [32, 64][trial % 2]
        kind = trial % 5
        x = rng.standard_normal(G).astype(np.float32)
        if kind == 1: x *= 1e-5                                       # subnormal halves
        if kind == 2: x = x * 100 + 3000
        if kind == 3: x[rng.integers(G)] *= 300                      # one outlier
        if kind == 4: x = np.round(x)                                 # many ties / equal values
        x = x.astype(np.float16)
        c, m = ref.quantize_group(x, bits)
        s = float(np.uint16(m & 0xffff).view(np.float16)); z = float(np.uint16(m >> 16).view(np.float16))
        xf = x.astype(np.float64)
        assert c.max() <= qmax and z == xf.min()
        assert c[xf.argmin()] == 0
        if xf.max() > xf.min():
            assert s >= (xf.max() - xf.min()) / qmax * (1 - 1e-7)        # rounded up
            assert s <= (xf.max() - xf.min()) / qmax * (1 + 2.0 ** -10) + 2.0 ** -24
            if s > 2.0 ** -14:
                assert c[xf.argmax()] == qmax
        else:
            assert s == 1.0 and (c == 0).all()
        assert np.all(np.abs(c * s + z - xf) <= 0.5001 * s)
    # negative zero is stored as +0
    x = np.zeros(32, np.float16); x[0] = -0.0
    assert ref.quantize_group(x, bits)[1] == 0x00003C00


def _read_words():
    cases, cur = {}, None
    for line in open(os.path.join(GOLD, "pack_words.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "case":
            shape = tuple(int(v) for v in t[3:6]) if len(t) >= 6 else (64, 64, 64)
            shape += (1 if t[-1] == "kpc" else 0,)
            cur = cases.setdefault((t[1], int(t[2]), shape), [])
        elif t[0] == "word":
            cur.append((t[1], int(t[2]), int(t[3], 16)))
    return cases


_GEN = {
    "k_dt_v_3dt": (lambda t, d: (d + t) % 4, lambda t, d: (3 * d + t) % 4),
    "k_dt_v_d5t": (lambda t, d: (d + t) % 16, lambda t, d: (d + 5 * t) % 16),
    "k_7dt_v_3d11t": (lambda t, d: np.where(d == 0, 0, np.where(d == 1, 255, (7 * d + t) % 256)),
                      lambda t, d: np.where(d == 0, 0, np.where(d == 1, 255, (3 * d + 11 * t) % 256))),
    # N = D = 128: the V code also depends on the token block, so that swapping block and column tile shows
    "n128_k_dt_v_3dt": (lambda t, d: (d + t) % 4, lambda t, d: (3 * d + t + t // 64) % 4),
    "n128_g32_zero": (lambda t, d: (d + t) % 16 + d // 32 + 4 * (t % 4),
                      lambda t, d: (d + 5 * t + t // 32) % 16 + 2 * (d // 32) + t % 2),
    "n32_k_dt_v_3dt": (lambda t, d: (d + t) % 4, lambda t, d: (3 * d + t + t // 16) % 4),
    "n32_g32_zero": (lambda t, d: (d + t) % 16 + d // 32 + 4 * (t % 4),
                     lambda t, d: (d + 5 * t + t // 8) % 16 + 2 * (d // 32) + t % 2),
    "n16_k_dt_v_3dt": (lambda t, d: (d + t) % 4, lambda t, d: (3 * d + t + t // 8) % 4),
    "n16_g32_zero": (lambda t, d: (d + t) % 16 + d // 32 + 4 * (t % 4),
                     lambda t, d: (d + 5 * t + t // 8) % 16 + 2 * (d // 32) + t % 2),
    "n8_k_dt_v_3dt": (lambda t, d: (d + t) % 4, lambda t, d: (3 * d + t) % 4),
    "n8_k_7dt_v_3d11t": (lambda t, d: np.where(d % 64 == 0, 0, np.where(d % 64 == 1, 255, (7 * d + t) % 256)),
                         lambda t, d: np.where(d % 64 == 0, 0, np.where(d % 64 == 1, 255, (3 * d + 11 * t) % 256))),
    "n128_kpc": (lambda t, d: (t + d) % 4 + d % 4 + 4 * (t // 64), lambda t, d: (3 * d + t + t // 64) % 4),
    "n128_k_7dt_v_3d11t": (lambda t, d: np.where(d % 64 == 0, 0, np.where(d % 64 == 1, 255, (7 * d + t) % 256)),
                           lambda t, d: np.where(d % 64 == 0, 0, np.where(d % 64 == 1, 255, (3 * d + 11 * t + t // 32) % 256))),
}


def test_pack_words_golden(ref):
    """A wrong bit position, word order, tile stride or area order moves these words."""
    cases = _read_words()
    assert any(shape[1] == 128 for (_, _, shape) in cases), "no case at the head size the library ships"
    assert any(shape[3] for (_, _, shape) in cases), "no per-channel case"
    for (name, bits, (N, D, G, kpc)), probes in cases.items():
        t, d = np.meshgrid(np.arange(N), np.arange(D), indexing="ij")
        cfg = ref.RefCfg(1, 1, 1, D, N, G, (bits, 16), 0, kpc)
        fk, fv = _GEN[name]
        blk = ref.pack_chunk(cfg, bits, fk(t, d).astype(np.float16), fv(t, d).astype(np.float16))
        cb, mb = N * D * bits // 8, N * (D // G) * 4
        vcb = max(N, 32 // bits, 8) * D * bits // 8                       # a chunk shorter than one V slice is stored as one slice
        areas = {"kcodes": 0, "kmeta": cb, "vcodes": cb + mb, "vmeta": cb + mb + vcb}
        assert blk.size == cb + vcb + 2 * mb
        assert any(N == 8 and b == 2 for (_, b, (N, _, _, _)) in cases), "no case with a padded V slice"
        for area, idx, val in probes:
            assert 4 * idx < {"kcodes": cb, "vcodes": vcb}.get(area, mb)
            got = int(blk[areas[area] + 4 * idx: areas[area] + 4 * idx + 4].view("<u4")[0])
            assert got == val, (name, area, idx, hex(got), hex(val))


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_pack_bit_coverage_is_a_bijection(ref, bits):
    """Every element owns b bits of the code area and no two elements share a bit."""
    for N, D, G in ((64, 128, 32), (32, 128, 64), (16, 128, 64), (8, 128, 32)):
        _bijection(ref, bits, N, D, G)


def _bijection(ref, bits, N, D, G):
    cfg = ref.RefCfg(1, 1, 1, D, N, G, (bits, 16), 0)
    cb, mb = N * D * bits // 8, N * (D // G) * 4
    vcb = max(N, 32 // bits, 8) * D * bits // 8
    tot_k = np.zeros(cb, np.uint8); tot_v = np.zeros(vcb, np.uint8)
    pop = lambda a: int(np.unpackbits(a).sum())
    for i in range(G):                                                  # element i of every group is the only non-zero one
        x = np.zeros((N, D), np.float16); x[:, i::G] = 1
        blk = ref.pack_chunk(cfg, bits, x, x)
        k, v = blk[:cb], blk[cb + mb: cb + mb + vcb]
        assert pop(k) == bits * N * (D // G) == pop(v)
        assert not (tot_k & k).any() and not (tot_v & v).any()
        tot_k |= k; tot_v |= v
    assert (tot_k == 0xFF).all()
    if vcb == cb:
        assert (tot_v == 0xFF).all()
    else:                                                               # 8 tokens at 2 bits: in-word indices 0..7 of every word
        assert vcb == 2 * cb and (tot_v.view("<u4") == 0x00FF00FF).all()


@pytest.mark.parametrize("bits,G,N", [(2, 64, 64), (4, 64, 64), (8, 64, 64), (2, 32, 64), (4, 32, 64), (16, 64, 64),
                                      (2, 64, 32), (4, 32, 32), (8, 64, 32), (16, 64, 32),
                                      (2, 64, 16), (4, 32, 16), (8, 64, 16), (16, 64, 16),
                                      (2, 32, 8), (4, 64, 8), (8, 32, 8), (16, 64, 8)])
def test_pack_decode_roundtrip_bound(ref, bits, G, N):
    """decode(pack(x)) stays within scale/2 of x for every element of K and V:
    the decoder reads each code, scale and zero from where the packer put it."""
    rng = np.random.default_rng(10 + bits)
    D = 128
    cfg = ref.RefCfg(1, 1, 1, D, N, G, (bits, 16), 0)
    Kc = rng.standard_normal((N, D)).astype(np.float32); Kc[:, [3, 50, 77, 120]] *= 10
    Kc = Kc.astype(np.float16); Vc = rng.standard_normal((N, D)).astype(np.float16)
    blk = ref.pack_chunk(cfg, bits, Kc, Vc)
    Kh, Vh = ref.decode_chunk(cfg, bits, blk)
    if bits == 16:
        assert blk.size == 2 * N * D * 2
        assert np.array_equal(blk.view(np.float16), np.concatenate([Kc.ravel(), Vc.ravel()]))
        assert np.array_equal(Kh, Kc.astype(np.float64)) and np.array_equal(Vh, Vc.astype(np.float64))
        return
    cb, mb = N * D * bits // 8, N * (D // G) * 4
    vcb = max(N, 32 // bits, 8) * D * bits // 8
    assert blk.size == cb + vcb + 2 * mb
    for x, xh, moff in [(Kc, Kh, cb), (Vc, Vh, cb + mb + vcb)]:
        meta = blk[moff: moff + mb].view("<u4").reshape(N, D // G)
        s = (meta & 0xffff).astype(np.uint16).view(np.float16).astype(np.float64)
        z = (meta >> 16).astype(np.uint16).view(np.float16).astype(np.float64)
        xg = x.astype(np.float64).reshape(N, D // G, G)
        assert np.array_equal(z, xg.min(-1))
        err = np.abs(xh.reshape(N, D // G, G) - xg)
        assert (err <= 0.5001 * s[..., None]).all()
        # decoded values sit on the grid zero + k*scale, k integer in [0, qmax]
        k = (xh.reshape(N, D // G, G) - z[..., None]) / s[..., None]
        assert np.allclose(k, np.round(k), atol=1e-9) and k.max() <= (1 << bits) - 1 + 1e-9 and k.min() >= 0


def test_block_sizes_offsets_and_capacity(ref):
    """Closed-form block sizes; arena = sum of block sizes in (b,h,c) order; capacity status."""
    cfg = ref.RefCfg(2, 3, 3, 128, 128, 64, (2, 4, 8, 16), 0)
    assert [ref.chunk_block_bytes(cfg, b) for b in (2, 4, 8, 16)] == [10240, 18432, 34816, 65536]
    cfg32 = ref.RefCfg(1, 1, 1, 128, 64, 32, (2, 4, 8, 16), 0)
    assert [ref.chunk_block_bytes(cfg32, b) for b in (2, 4, 8, 16)] == [6144, 10240, 18432, 32768]
    # small chunks: 2 * (N*D*b/8 + N*(D/G)*4), except 8 tokens at 2 bits, whose V codes take a whole slice of 16 tokens
    cfg16 = ref.RefCfg(1, 1, 1, 128, 16, 64, (2, 4, 8, 16), 0)
    assert [ref.chunk_block_bytes(cfg16, b) for b in (2, 4, 8, 16)] == [1280, 2304, 4352, 8192]
    cfg8 = ref.RefCfg(1, 1, 1, 128, 8, 32, (2, 4, 8, 16), 0)
    assert [ref.chunk_block_bytes(cfg8, b) for b in (2, 4, 8, 16)] == [256 + 128 + 512 + 128, 1280, 2304, 4096]
    rng = np.random.default_rng(4)
    C = 5
    K = rng.standard_normal((2, 3, C * 128 + 7, 128)).astype(np.float16)
    V = rng.standard_normal(K.shape).astype(np.float16)
    expert = rng.integers(0, 4, (6, C)).astype(np.uint8)
    sizes = np.array([10240, 18432, 34816, 65536], np.uint64)[expert]
    arena = np.zeros(int(sizes.sum()) + 512, np.uint8)
    used = np.array([300], np.uint64)                                   # start is rounded up to 512
    off = np.zeros((6, C), np.uint64)
    assert ref.quantize_pack(cfg, K, V, 0, C, expert, arena, used, off) == 0
    want = 512 + np.concatenate([[0], np.cumsum(sizes.ravel())[:-1]]).reshape(6, C)
    assert np.array_equal(off, want.astype(np.uint64)) and used[0] == 512 + sizes.sum()
    # each block equals the stand-alone packing of its chunk
    for u, c in [(0, 0), (3, 2), (5, 4)]:
        b, h = divmod(u, 3)
        bits = cfg.expert_bits[expert[u, c]]
        blk = ref.pack_chunk(cfg, bits, K[b, h, c * 128:(c + 1) * 128], V[b, h, c * 128:(c + 1) * 128])
        assert np.array_equal(arena[int(off[u, c]): int(off[u, c]) + blk.size], blk)
    # too small an arena: status set, nothing else written
    used2 = np.array([0], np.uint64)
    small = np.zeros(int(sizes.sum()) - 256, np.uint8)
    off2 = np.full((6, C), 77, np.uint64)
    st = np.zeros(1, np.int32)
    assert ref.quantize_pack(cfg, K, V, 0, C, expert, small, used2, off2, st) == -3
    assert used2[0] == 0 and (off2 == 77).all() and not small.any()
    # a non-zero status on entry makes the call a no-op
    assert ref.quantize_pack(cfg, K, V, 0, C, expert, arena, used2, off2, st) == -3 and used2[0] == 0
    # an expert index >= M is reported through the status word
    bad = expert.copy(); bad[2, 1] = 4
    st[0] = 0
    assert ref.quantize_pack(cfg, K, V, 0, C, bad, arena, used2, off2, st) == -1 and used2[0] == 0


def test_sanity_numbers_from_the_paper():
    """Sec. 4.1: router parameters take about 1.6 KB; Sec. 1: the KV cache of
    Llama2-13B reaches about 100 GB at 128k context."""
    D, M = 128, 3
    assert abs((2 * D * M + M * M) * 2 - 1600) < 100                    # 1554 B with three experts in fp16
    kv = 40 * 40 * 128 * 2 * 2 * 131072                                  # layers * heads * dim * (K,V) * bytes * tokens
    assert 95e9 < kv < 115e9


# ----------------------------------------------------------------------------
# Decode attention
# ----------------------------------------------------------------------------

def _sdpa(q, K, V, scale, rep):
    """torch fp64 scaled_dot_product_attention; q [B,Hq,D], K/V [B,Hkv,S,D]."""
    qt = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    Kt = torch.from_numpy(K.astype(np.float64)).repeat_interleave(rep, 1)
    Vt = torch.from_numpy(V.astype(np.float64)).repeat_interleave(rep, 1)
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=scale)[:, :, 0].numpy()


def _packed(ref, cfg, K, V, expert, C):
    arena = np.zeros(int(ref.chunk_block_bytes(cfg, 16)) * expert.shape[0] * max(C, 1) + 256, np.uint8)
    used = np.zeros(1, np.uint64); off = np.zeros(expert.shape, np.uint64)
    assert ref.quantize_pack(cfg, K, V, 0, C, expert, arena, used, off) == 0
    return arena, off


@pytest.mark.parametrize("B,Hq,Hkv,S,N", [(1, 4, 4, 256, 64), (2, 8, 2, 64 * 3 + 17, 64), (1, 2, 1, 5, 64),
                                          (1, 4, 2, 16 * 5 + 11, 16), (2, 2, 2, 8 * 9 + 7, 8)])
def test_attention_all_16bit_equals_unquantised(ref, B, Hq, Hkv, S, N):
    """With only the FP16 expert the path must reproduce plain attention
    (residual rows included, GQA head mapping included)."""
    rng = np.random.default_rng(S)
    D = 128
    K = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    V = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    C, T = S // N, S % N
    cfg = ref.RefCfg(B, Hq, Hkv, D, N, 64, (2, 16), 1)
    expert = np.ones((B * Hkv, max(C, 1)), np.uint8)
    arena, off = _packed(ref, cfg, K, V, expert, C)
    Kt = np.zeros((B, Hkv, N, D), np.float16); Vt = np.zeros_like(Kt)
    Kt[:, :, :T] = K[:, :, C * N:]; Vt[:, :, :T] = V[:, :, C * N:]
    scale = 1 / math.sqrt(D)
    out = ref.decode_attn(cfg, q, arena, off, expert, C, Kt, Vt, T, scale)
    want = _sdpa(q, K, V, scale, Hq // Hkv)
    assert np.abs(out - want).max() < 1e-12


@pytest.mark.parametrize("N,C,T", [(64, 6, 9), (16, 13, 5), (8, 21, 7)])
def test_attention_quantised_is_attention_over_decoded_cache(ref, N, C, T):
    """Mixed bit-widths: the result equals library attention over the decoded K^, V^."""
    rng = np.random.default_rng(9)
    B, Hq, Hkv, D = 2, 4, 2, 128
    S = C * N + T
    K = rng.standard_normal((B, Hkv, S, D)).astype(np.float32); K[..., [1, 2, 3, 4]] *= 10
    K = K.astype(np.float16); V = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    cfg = ref.RefCfg(B, Hq, Hkv, D, N, 32, (2, 4, 8, 16), 1)
    expert = rng.integers(0, 4, (B * Hkv, C)).astype(np.uint8)
    arena, off = _packed(ref, cfg, K, V, expert, C)
    Kh = K.astype(np.float64).copy(); Vh = V.astype(np.float64).copy()
    for u in range(B * Hkv):
        for c in range(C):
            bits = cfg.expert_bits[expert[u, c]]
            blk = arena[int(off[u, c]): int(off[u, c]) + ref.chunk_block_bytes(cfg, bits)]
            Kh[u // Hkv, u % Hkv, c * N:(c + 1) * N], Vh[u // Hkv, u % Hkv, c * N:(c + 1) * N] = ref.decode_chunk(cfg, bits, blk)
    Kt = np.zeros((B, Hkv, N, D), np.float16); Vt = np.zeros_like(Kt)
    Kt[:, :, :T] = K[:, :, C * N:]; Vt[:, :, :T] = V[:, :, C * N:]
    out = ref.decode_attn(cfg, q, arena, off, expert, C, Kt, Vt, T, 0.11)
    want = _sdpa(q, Kh, Vh, 0.11, 2)
    assert np.abs(out - want).max() < 1e-12
    # quantisation did change something (the test is not vacuous)
    assert np.abs(want - _sdpa(q, K, V, 0.11, 2)).max() > 1e-4


def test_attention_special_cases(ref):
    rng = np.random.default_rng(12)
    N, D = 64, 128
    cfg = ref.RefCfg(1, 2, 1, D, N, 64, (4, 16), 0)
    q = rng.standard_normal((1, 2, D)).astype(np.float16)
    # S = 1 (a single residual row): the output is that row of V
    Kt = rng.standard_normal((1, 1, N, D)).astype(np.float16); Vt = rng.standard_normal((1, 1, N, D)).astype(np.float16)
    out = ref.decode_attn(cfg, q, None, None, None, 0, Kt, Vt, 1, 0.3)
    assert np.allclose(out[0, 0], Vt[0, 0, 0].astype(np.float64), atol=0, rtol=1e-15)
    assert np.allclose(out[0, 1], Vt[0, 0, 0].astype(np.float64), atol=0, rtol=1e-15)
    # identical keys: uniform weights, output = mean of the decoded values
    K = np.tile(rng.standard_normal((1, 1, 1, D)).astype(np.float16), (1, 1, 2 * N, 1))
    V = rng.standard_normal((1, 1, 2 * N, D)).astype(np.float16)
    expert = np.zeros((1, 2), np.uint8)
    arena, off = _packed(ref, cfg, K, V, expert, 2)
    out = ref.decode_attn(cfg, q, arena, off, expert, 2, None, None, 0, 0.2)
    Vh = np.concatenate([ref.decode_chunk(cfg, 4, arena[int(off[0, c]):])[1] for c in range(2)])
    assert np.allclose(out[0, 0], Vh.mean(0), rtol=1e-12, atol=1e-14)
    # adding a constant to all scores (q -> q + k0-orthogonal shift is not available in fp16, so
    # scale both ways instead): scale 0 gives the plain mean whatever the keys are
    K2 = rng.standard_normal((1, 1, 2 * N, D)).astype(np.float16)
    arena, off = _packed(ref, cfg, K2, V, expert, 2)
    out0 = ref.decode_attn(cfg, q, arena, off, expert, 2, None, None, 0, 0.0)
    Vh = np.concatenate([ref.decode_chunk(cfg, 4, arena[int(off[0, c]):])[1] for c in range(2)])
    assert np.allclose(out0[0, 1], Vh.mean(0), rtol=1e-12, atol=1e-14)
    # a huge scale picks the single best key of each query
    outb = ref.decode_attn(cfg, q, arena, off, expert, 2, None, None, 0, 50.0)
    Kh = np.concatenate([ref.decode_chunk(cfg, 4, arena[int(off[0, c]):])[0] for c in range(2)])
    for hq in range(2):
        best = (Kh @ q[0, hq].astype(np.float64)).argmax()
        assert np.allclose(outb[0, hq], Vh[best], atol=1e-6)


# ----------------------------------------------------------------------------
# keys quantised per channel (k_per_channel)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("bits,G,N", [(2, 64, 128), (4, 32, 64), (8, 64, 64), (2, 32, 32)])
def test_per_channel_keys_roundtrip_and_meta(ref, bits, G, N):
    """Groups run along tokens: zero = minimum of the G tokens of a dim, |x - x^| <= scale/2, meta at [token group][dim];
    the values and the places of the key codes are untouched by the flag."""
    rng = np.random.default_rng(bits + N)
    D = 128
    cfg = ref.RefCfg(1, 1, 1, D, N, G, (bits, 16), 0, 1)
    cfg0 = ref.RefCfg(1, 1, 1, D, N, G, (bits, 16), 0, 0)
    Kc = rng.standard_normal((N, D)).astype(np.float32); Kc[:, [3, 50, 77, 120]] *= 10
    Kc = Kc.astype(np.float16); Vc = rng.standard_normal((N, D)).astype(np.float16)
    blk = ref.pack_chunk(cfg, bits, Kc, Vc); blk0 = ref.pack_chunk(cfg0, bits, Kc, Vc)
    cb, mb = N * D * bits // 8, N * (D // G) * 4
    assert blk.size == blk0.size == 2 * (cb + mb)
    assert np.array_equal(blk[cb + mb:], blk0[cb + mb:])                 # the V half does not depend on the flag
    Kh, Vh = ref.decode_chunk(cfg, bits, blk)
    meta = blk[cb:cb + mb].view("<u4").reshape(N // G, D)
    s = (meta & 0xffff).astype(np.uint16).view(np.float16).astype(np.float64)
    z = (meta >> 16).astype(np.uint16).view(np.float16).astype(np.float64)
    xg = Kc.astype(np.float64).reshape(N // G, G, D)
    assert np.array_equal(z, xg.min(1))
    rng_ = xg.max(1) - xg.min(1)
    assert np.all(s >= rng_ / ((1 << bits) - 1) * (1 - 1e-7)) and np.all(s <= rng_ / ((1 << bits) - 1) * (1 + 2.0 ** -10) + 2.0 ** -24)
    err = np.abs(Kh.reshape(N // G, G, D) - xg)
    assert (err <= 0.5001 * s[:, None, :]).all()
    # every group is what the (pinned) group quantiser makes of the G tokens of the dim; codes sit where the per-token layout puts them
    for tg, d in [(0, 0), (N // G - 1, 50), (0, 127)]:
        codes, m = ref.quantize_group(np.ascontiguousarray(Kc[tg * G:(tg + 1) * G, d]), bits)
        assert int(meta[tg, d]) == m
        k = np.round((Kh[tg * G:(tg + 1) * G, d] - z[tg, d]) / s[tg, d]).astype(np.int64)
        assert np.array_equal(k, codes.astype(np.int64))
    # the outlier channels no longer blow up the error of their neighbours: per channel beats per token on this K
    Kh0, _ = ref.decode_chunk(cfg0, bits, blk0)
    if N >= 64:
        assert np.abs(Kh - Kc).mean() < np.abs(Kh0 - Kc).mean()


def test_per_channel_attention_is_attention_over_the_decoded_cache(ref):
    rng = np.random.default_rng(21)
    B, Hq, Hkv, N, G, C, T = 1, 2, 2, 64, 64, 5, 9
    cfg = ref.RefCfg(B, Hq, Hkv, 128, N, G, (2, 4, 8, 16), 0, 1)
    S = C * N + T
    K = rng.standard_normal((B, Hkv, S, 128)).astype(np.float16); V = rng.standard_normal((B, Hkv, S, 128)).astype(np.float16)
    q = rng.standard_normal((B, Hq, 128)).astype(np.float16)
    expert = rng.integers(0, 4, (B * Hkv, C)).astype(np.uint8)
    cap = C * B * Hkv * 32768 + 4096
    arena = np.zeros(cap, np.uint8); used = np.zeros(1, np.uint64); off = np.zeros((B * Hkv, C), np.uint64)
    assert ref.quantize_pack(cfg, K, V, 0, C, expert, arena, used, off) == 0
    Kt = np.zeros((B, Hkv, N, 128), np.float16); Vt = np.zeros_like(Kt)
    Kt[:, :, :T] = K[:, :, C * N:]; Vt[:, :, :T] = V[:, :, C * N:]
    o = ref.decode_attn(cfg, q, arena, off, expert, C, Kt, Vt, T, 0.1)
    for u in range(B * Hkv):
        Kh = np.zeros((S, 128)); Vh = np.zeros((S, 128))
        for c in range(C):
            bits = (2, 4, 8, 16)[expert[u, c]]
            nb = ref.chunk_block_bytes(cfg, bits)
            kk, vv = ref.decode_chunk(cfg, bits, arena[int(off[u, c]):int(off[u, c]) + nb])
            Kh[c * N:(c + 1) * N] = kk; Vh[c * N:(c + 1) * N] = vv
        Kh[C * N:] = Kt[0, u, :T]; Vh[C * N:] = Vt[0, u, :T]
        sc = 0.1 * (Kh @ q[0, u].astype(np.float64)); p = np.exp(sc - sc.max()); p /= p.sum()
        assert np.allclose(o[0, u], p @ Vh, rtol=1e-10, atol=1e-12)


def test_several_queries_are_causal_attention_over_the_new_tokens(ref):
    """All-16-bit cache: Q new tokens against torch fp64 attention over [cache + residual] with a causal mask on the
    new tokens (query t sees everything up to and including its own row)."""
    rng = np.random.default_rng(31)
    B, Hq, Hkv, N, C, T, Q = 2, 4, 2, 64, 3, 21, 4
    cfg = ref.RefCfg(B, Hq, Hkv, 128, N, 64, (16,), 0)
    S = C * N + T
    K = rng.standard_normal((B, Hkv, S, 128)).astype(np.float16); V = rng.standard_normal((B, Hkv, S, 128)).astype(np.float16)
    q = rng.standard_normal((B, Q, Hq, 128)).astype(np.float16)
    expert = np.zeros((B * Hkv, C), np.uint8)
    arena = np.zeros(B * Hkv * C * 2 * N * 128 * 2 + 4096, np.uint8); used = np.zeros(1, np.uint64); off = np.zeros((B * Hkv, C), np.uint64)
    assert ref.quantize_pack(cfg, K, V, 0, C, expert, arena, used, off) == 0
    Kt = np.zeros((B, Hkv, N, 128), np.float16); Vt = np.zeros_like(Kt)
    Kt[:, :, :T] = K[:, :, C * N:]; Vt[:, :, :T] = V[:, :, C * N:]
    o = ref.decode_attn_multi(cfg, q, arena, off, expert, C, Kt, Vt, T, 0.11)
    rep = Hq // Hkv
    Kx = torch.from_numpy(K.astype(np.float64)).repeat_interleave(rep, 1); Vx = torch.from_numpy(V.astype(np.float64)).repeat_interleave(rep, 1)
    qx = torch.from_numpy(q.astype(np.float64)).permute(0, 2, 1, 3)                           # [B, Hq, Q, D]
    mask = torch.ones(Q, S, dtype=torch.bool)
    for t in range(Q):
        mask[t, S - (Q - 1 - t):] = False
    want = torch.nn.functional.scaled_dot_product_attention(qx, Kx, Vx, attn_mask=mask, scale=0.11).permute(0, 2, 1, 3).numpy()
    assert np.allclose(o, want, rtol=1e-9, atol=1e-12)
