"""GPU parity of moqae_router_loss_grad (the router fine-tuning loss of Sec. 3.3, Eq. (3)-(5), and its gradient)
against the CPU oracle (binary64 given the binary32 top-1 decision)."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import test_gpu_parity as T                                              # noqa: E402  (helpers only)

mq = T.mq
BITS = (2, 4, 8, 16)
# binary32 forward / backward per row and sums over up to ~1e5 rows added in no fixed order, against binary64:
# relative to the largest entry of each gradient array
GRAD_TOL, LOSS_TOL = 2e-4, 2e-5


@pytest.mark.parametrize("B,Hkv,S,t0,t1,M,std,use_bias,defaults", [
    (1, 8, 2048, 0, 2048, 4, 0.02, False, True),      # the tiny workload's shape, router at its initial scale
    (2, 3, 700, 13, 650, 4, 0.3, True, False),        # ragged token range, partial last tile
    (1, 2, 200, 0, 200, 3, 0.3, True, False),
    (3, 1, 130, 64, 130, 8, 0.2, False, False),
    (1, 1, 64, 0, 1, 1, 0.3, False, True),            # one row, one expert
])
def test_router_loss_grad(mq, ref, B, Hkv, S, t0, t1, M, std, use_bias, defaults):
    print(f"\n[gpu-case] train B={B} Hkv={Hkv} S={S} [{t0},{t1}) M={M}", file=sys.stderr, flush=True)
    rng = np.random.default_rng(S + M)
    bits = BITS[:M] if M <= 4 else (2, 2, 4, 4, 8, 8, 16, 16)
    cfg, rcfg = T._cfgs(mq, ref, B, Hkv, Hkv, 64, 64, bits, 0)
    K, _ = T._rand_kv(rng, B, Hkv, S)
    W1 = (rng.standard_normal((128, M)) * std).astype(np.float16)
    W2 = (rng.standard_normal((128, M)) * std).astype(np.float16)
    W3 = (rng.standard_normal((M, M)) * (0.5 if std > 0.1 else 0.02) + (np.eye(M) if std > 0.1 else 0)).astype(np.float16)
    bias = (rng.standard_normal(M) * 0.1).astype(np.float32) if use_bias else None
    nll = rng.uniform(1.5, 3.0, B).astype(np.float32)
    pm = np.array([1.0 / b for b in bits], np.float32)
    pe = np.array([16.0 / b for b in bits], np.float32) if defaults else np.array([b / 16.0 for b in bits], np.float32)
    lam = 0.5
    l_ref, g1, g2, g3, gb = ref.router_loss_grad(rcfg, K, t0, t1, W1, W2, W3, bias, nll, pm, pe, lam)
    dev = "cuda"
    loss = torch.full((3,), 7.0, dtype=torch.float32, device=dev)              # outputs are overwritten
    dW1 = torch.full((128, M), 7.0, dtype=torch.float32, device=dev); dW2 = torch.full_like(dW1, 7.0)
    dW3 = torch.full((M, M), 7.0, dtype=torch.float32, device=dev); db = torch.full((M,), 7.0, dtype=torch.float32, device=dev)
    mq.router_loss_grad(cfg, T._dev(K), t0, t1, T._dev(W1), T._dev(W2), T._dev(W3), None if bias is None else T._dev(bias),
                        T._dev(nll), None if defaults else pm, None if defaults else pe, lam, loss, dW1, dW2, dW3, db)
    torch.cuda.synchronize()
    l = loss.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(l - l_ref) <= LOSS_TOL * np.abs(l_ref).max()), (l, l_ref)
    for name, g, r in (("dW1", dW1, g1), ("dW2", dW2, g2), ("dW3", dW3, g3), ("dbias", db, gb)):
        got = g.cpu().numpy().astype(np.float64)
        scale = max(np.abs(r).max(), 1e-30)
        assert np.abs(got - r).max() <= GRAD_TOL * scale, (name, np.abs(got - r).max() / scale)
