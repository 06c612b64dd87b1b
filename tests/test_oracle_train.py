"""Pins of the oracle's router fine-tuning loss and gradient (Sec. 3.3, Eq. (3)-(5)) to things other than itself:
closed-form special cases of the loss, and the gradient against central finite differences of the loss."""
import numpy as np
import pytest

BITS = (2, 4, 8, 16)


def _case(ref, seed=0, B=2, Hkv=2, S=24, M=4, std=0.3):
    rng = np.random.default_rng(seed)
    cfg = ref.RefCfg(B, Hkv, Hkv, 128, 32, 64, BITS[:M], 0)
    K = rng.standard_normal((B, Hkv, S, 128), dtype=np.float32).astype(np.float16)
    W1 = (rng.standard_normal((128, M)) * std).astype(np.float16)
    W2 = (rng.standard_normal((128, M)) * std).astype(np.float16)
    W3 = (rng.standard_normal((M, M)) * 0.5 + np.eye(M)).astype(np.float16)
    bias = (rng.standard_normal(M) * 0.1).astype(np.float32)
    nll = rng.uniform(1.5, 3.0, B).astype(np.float32)
    pm = np.array([1.0 / b for b in BITS[:M]], np.float32); pe = np.array([16.0 / b for b in BITS[:M]], np.float32)
    return cfg, K, W1, W2, W3, bias, nll, pm, pe


def test_one_expert_gives_a_constant_loss_and_no_gradient(ref):
    cfg, K, W1, W2, W3, bias, nll, pm, pe = _case(ref, M=1)
    loss, dW1, dW2, dW3, db = ref.router_loss_grad(cfg, K, 0, 24, W1, W2, W3, bias, nll, pm, pe, 0.3)
    # p = 1 for the only expert: L_model = mean over tokens of L_nll / B_0, L_mem = 16 / B_0
    assert abs(loss[1] - nll.astype(np.float64).mean() * 0.5) < 1e-12 and abs(loss[2] - 8.0) < 1e-12
    assert abs(loss[0] - (0.3 * loss[1] + 0.7 * loss[2])) < 1e-12
    for g in (dW1, dW2, dW3, db):
        assert np.abs(g).max() < 1e-15


def test_uniform_probabilities(ref):
    """W3 = 0 and no bias: every logit is 0, p = 1/M, the first expert wins the tie: L = (1/M) * its penalties."""
    cfg, K, W1, W2, W3, bias, nll, pm, pe = _case(ref, seed=1)
    W3 = np.zeros((4, 4), np.float16)
    loss, *_ = ref.router_loss_grad(cfg, K, 0, 24, W1, W2, W3, None, nll, pm, pe, 0.5)
    assert abs(loss[1] - 0.25 * nll.astype(np.float64).mean() * float(pm[0])) < 1e-12
    assert abs(loss[2] - 0.25 * float(pe[0])) < 1e-12


def test_lambda_limits_and_linearity_in_nll(ref):
    cfg, K, W1, W2, W3, bias, nll, pm, pe = _case(ref, seed=2)
    l0, g0, *_ = ref.router_loss_grad(cfg, K, 0, 24, W1, W2, W3, bias, nll, pm, pe, 0.0)
    l1, g1, *_ = ref.router_loss_grad(cfg, K, 0, 24, W1, W2, W3, bias, nll, pm, pe, 1.0)
    lh, gh, *_ = ref.router_loss_grad(cfg, K, 0, 24, W1, W2, W3, bias, nll, pm, pe, 0.25)
    assert abs(l0[0] - l0[2]) < 1e-12 and abs(l1[0] - l1[1]) < 1e-12
    assert np.allclose(gh, 0.25 * g1 + 0.75 * g0, rtol=1e-12, atol=1e-15)        # the loss is linear in lambda
    l2, g2, *_ = ref.router_loss_grad(cfg, K, 0, 24, W1, W2, W3, bias, 2 * nll, pm, pe, 1.0)
    assert abs(l2[1] - 2 * l1[1]) < 1e-12 and np.allclose(g2, 2 * g1, rtol=1e-12)  # and L_model in L_nll
    # a sub-range of tokens is the mean over that sub-range
    la, *_ = ref.router_loss_grad(cfg, K, 0, 12, W1, W2, W3, bias, nll, pm, pe, 0.5)
    lb, *_ = ref.router_loss_grad(cfg, K, 12, 24, W1, W2, W3, bias, nll, pm, pe, 0.5)
    lf, *_ = ref.router_loss_grad(cfg, K, 0, 24, W1, W2, W3, bias, nll, pm, pe, 0.5)
    assert np.allclose(lf, 0.5 * (la + lb), rtol=1e-12)


def test_gradient_against_finite_differences(ref):
    """Central differences of the oracle's loss in the fp16 weights (steps of a few fp16 ulps) and in the bias."""
    cfg, K, W1, W2, W3, bias, nll, pm, pe = _case(ref, seed=3, S=16)
    lam = 0.4
    args = lambda w1, w2, w3, b: (cfg, K, 0, 16, w1, w2, w3, b, nll, pm, pe, lam)
    loss, dW1, dW2, dW3, db = ref.router_loss_grad(*args(W1, W2, W3, bias))
    rng = np.random.default_rng(0)
    checked = 0
    for name, Wm, g in (("W1", W1, dW1), ("W2", W2, dW2), ("W3", W3, dW3)):
        for _ in range(12):
            idx = tuple(int(rng.integers(n)) for n in Wm.shape)
            w0 = np.float64(Wm[idx])
            hi = Wm.copy(); lo = Wm.copy()
            step = 8 * abs(float(np.spacing(Wm[idx])))                      # eight fp16 ulps: exactly representable
            hi[idx] = np.float16(w0 + step); lo[idx] = np.float16(w0 - step)
            assert float(hi[idx]) - float(lo[idx]) == 2 * step
            mk = lambda Wx: [Wx if name == n else Wo for n, Wo in (("W1", W1), ("W2", W2), ("W3", W3))]
            lp = ref.router_loss_grad(*args(*mk(hi), bias))[0][0]
            lm = ref.router_loss_grad(*args(*mk(lo), bias))[0][0]
            fd = (lp - lm) / (2 * step)
            # a top-1 flip between the two points would show as a jump: the second difference stays small when none happened
            if abs(lp - 2 * loss[0] + lm) > 1e-4 * abs(loss[0]):
                continue
            assert abs(fd - g[idx]) <= 2e-3 * max(abs(g[idx]), np.abs(g).max() * 1e-2), (name, idx, fd, g[idx])
            checked += 1
    for k in range(4):
        e = np.zeros(4, np.float32); e[k] = 2.0 ** -9
        lp = ref.router_loss_grad(*args(W1, W2, W3, bias + e))[0][0]
        lm = ref.router_loss_grad(*args(W1, W2, W3, bias - e))[0][0]
        assert abs((lp - lm) / 2.0 ** -8 - db[k]) <= 2e-3 * np.abs(db).max(), k
        checked += 1
    assert checked >= 30
