"""Pins for the oracle's SliM-LLM+ functions (Sec. 3.4, Sec. 4, App. B: SBA's widths, no SQC, learnable weight
clipping trained with AdamW).  The paper names the method it borrows and no more, so the forward pass is a stated
reading; what is pinned here is (i) that full clipping strength reproduces Eq. 1, (ii) that the hand-written
derivatives are those of that forward pass under the straight-through rule (PyTorch autograd on the CPU builds them
independently from the forward pass alone), (iii) that the optimiser step is AdamW (torch.optim on the CPU), and
(iv) that the whole training loop equals the autograd + torch.optim loop of the same forward pass."""
import numpy as np
import pytest
import torch

from oracle import slim_oracle as orc


def _case(seed, n=6, m=32, beta=8, t=40):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((n, m)) * 0.05
    X = rng.standard_normal((m, t)) * rng.lognormal(0, 0.5, m)[:, None]
    return W, X @ X.T, t


def _torch_forward(Wt, gam, bet, bits, beta):
    """The forward pass of lwc_forward written again in PyTorch, rounding with the straight-through rule."""
    n, m = Wt.shape
    k = m // beta
    Wg = Wt.reshape(n, k, beta)
    Q = torch.tensor(2.0 ** bits.astype(np.float64) - 1.0)[None, :]
    hi = torch.sigmoid(gam) * Wg.max(2).values
    lo = torch.sigmoid(bet) * Wg.min(2).values
    delta = (hi - lo) / Q
    ste = lambda x: x + (torch.round(x) - x).detach()
    z = -ste(lo / delta)
    u = ste(Wg / delta[:, :, None]) + z[:, :, None]
    q = torch.clamp(u, min=torch.zeros_like(u), max=Q[:, :, None].expand_as(u))
    return (delta[:, :, None] * (q - z[:, :, None])).reshape(n, m)


def test_full_strength_is_eq1():
    W, G, t = _case(1)
    bits = np.array([1, 2, 3, 4], dtype=np.uint8)
    big = np.full((6, 4), 40.0)                            # sigmoid(40) == 1 in float64
    f = orc.lwc_forward(W, big, big, bits, 8)
    ref = orc.rtn_fakequant(W, bits, 8, q1_mode=orc.Q1_AFFINE)
    assert np.array_equal(f["What"], ref)
    for i in range(6):
        for g in range(4):
            d0, z0 = orc.minmax_params(W[i, g * 8:(g + 1) * 8], int(bits[g]))
            assert f["scale"][i, g] == d0 and f["zero"][i, g] == z0
    assert f["codes"].max() <= 15 and np.all(f["codes"][:, :8] <= 1)
    # an all-zero (row, group) has nothing to clip
    W0 = W.copy()
    W0[2, 8:16] = 0.0
    f0 = orc.lwc_forward(W0, big, big, bits, 8)
    assert f0["scale"][2, 1] == 1.0 and f0["zero"][2, 1] == 0.0 and np.all(f0["What"][2, 8:16] == 0.0)


@pytest.mark.parametrize("seed", [2, 3, 4])
def test_derivatives_are_those_of_the_forward_pass(seed):
    W, G, t = _case(seed)
    rng = np.random.default_rng(seed + 100)
    bits = np.array([1, 2, 3, 2], dtype=np.uint8)
    gam, bet = rng.uniform(-1.0, 4.0, (6, 4)), rng.uniform(-1.0, 4.0, (6, 4))
    loss, gg, gb, f = orc.lwc_loss_and_grads(W, G, t, gam, bet, bits, 8)
    assert (~f["inside"]).any()                            # some weights are clipped: both branches are exercised
    tg = torch.tensor(gam, requires_grad=True)
    tb = torch.tensor(bet, requires_grad=True)
    Wt = torch.tensor(W)
    D = _torch_forward(Wt, tg, tb, bits, 8) - Wt
    L = (D * (D @ torch.tensor(G))).sum() / (6 * t)
    L.backward()
    assert loss == pytest.approx(L.item(), rel=1e-13)
    assert np.allclose(gg, tg.grad.numpy(), rtol=1e-10, atol=1e-18)
    assert np.allclose(gb, tb.grad.numpy(), rtol=1e-10, atol=1e-18)
    # the loss is the mean squared error of the layer's outputs (Eq. 3)
    X = np.linalg.cholesky(G + 1e-9 * np.eye(32))           # any X with X X^T = G gives the same loss
    assert loss == pytest.approx(np.sum(((W - f["What"]) @ X) ** 2) / (6 * t), rel=1e-6)


def test_adamw_step_is_torch_adamw():
    rng = np.random.default_rng(5)
    p0 = rng.standard_normal((3, 4))
    grads = [rng.standard_normal((3, 4)) for _ in range(5)]
    p, m1, v = p0.copy(), np.zeros((3, 4)), np.zeros((3, 4))
    tp = torch.tensor(p0.copy(), requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=1e-2, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0)
    for it, g in enumerate(grads, 1):
        orc.adamw_step(p, g, m1, v, it, 1e-2, 0.9, 0.999, 1e-8)
        tp.grad = torch.tensor(g)
        opt.step()
        assert np.allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-15)
    # the first step moves every parameter by lr against the sign of its derivative
    p1, m1, v = p0.copy(), np.zeros((3, 4)), np.zeros((3, 4))
    orc.adamw_step(p1, grads[0], m1, v, 1, 1e-2, 0.9, 0.999, 1e-8)
    assert np.allclose(p1 - p0, -1e-2 * np.sign(grads[0]), rtol=1e-6)


def test_training_loop_equals_autograd_with_torch_adamw():
    W, G, t = _case(6, n=8, m=48, beta=16, t=64)
    bits = np.array([1, 2, 3], dtype=np.uint8)
    steps = 12
    out = orc.lwc_quantize(W, G, t, bits, 16, steps=steps, lr=1e-2)
    tg = torch.full((8, 3), 4.0, dtype=torch.float64, requires_grad=True)
    tb = torch.full((8, 3), 4.0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tg, tb], lr=1e-2, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0)
    Wt, Gt = torch.tensor(W), torch.tensor(G)
    curve = []
    for _ in range(steps):
        opt.zero_grad()
        D = _torch_forward(Wt, tg, tb, bits, 16) - Wt
        L = (D * (D @ Gt)).sum() / (8 * t)
        curve.append(L.item())
        L.backward()
        opt.step()
    assert np.allclose(out["loss_curve"][:steps], curve, rtol=1e-9)
    assert np.allclose(out["gamma"], tg.detach().numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(out["beta_p"], tb.detach().numpy(), rtol=1e-9, atol=1e-12)
    with torch.no_grad():
        assert np.allclose(out["What"], _torch_forward(Wt, tg, tb, bits, 16).numpy(), rtol=0, atol=1e-12)
    # training lowers the layer-output error, and the start of the curve is the loss of the start values
    assert out["loss_curve"][-1] < out["loss_curve"][0]
    l0, _, _, _ = orc.lwc_loss_and_grads(W, G, t, np.full((8, 3), 4.0), np.full((8, 3), 4.0), bits, 16)
    assert out["loss_curve"][0] == l0
