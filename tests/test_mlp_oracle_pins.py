"""Pins of the dense-step oracle: torch autograd in fp64 (library routine) for the loss and every gradient,
torch.optim.SGD for the update, a finite difference on a toy net, and the size of the bf16 effect."""
import numpy as np
import torch

from oracle import mlp_oracle as M


def _net(seed, widths):
    rng = np.random.default_rng(seed)
    Ws = [(rng.standard_normal((i, o)) * np.sqrt(2.0 / i)).astype(np.float32) for i, o in zip(widths[:-1], widths[1:])]
    bs = [(rng.standard_normal(o) * 0.1).astype(np.float32) for o in widths[1:]]
    return Ws, bs


def _data(seed, B, P, Dn):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, P)).astype(np.float32) * 0.3, rng.standard_normal((B, Dn)).astype(np.float32),
            (rng.random(B) < 0.3).astype(np.float32))


def _torch_ref(Ws, bs, pooled, dense, y, mean):
    tW = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in Ws]
    tb = [torch.tensor(b, dtype=torch.float64, requires_grad=True) for b in bs]
    tp = torch.tensor(pooled, dtype=torch.float64, requires_grad=True)
    h = torch.cat([tp, torch.tensor(dense, dtype=torch.float64)], dim=1)
    for l in range(len(Ws) - 1):
        h = torch.relu(h @ tW[l] + tb[l])
    z = (h @ tW[-1] + tb[-1]).reshape(-1)
    loss = torch.nn.functional.binary_cross_entropy_with_logits(z, torch.tensor(y, dtype=torch.float64),
                                                                 reduction="mean" if mean else "sum")
    loss.backward()
    return loss.item(), tp.grad.numpy(), [w.grad.numpy() for w in tW], [b.grad.numpy() for b in tb], tW, tb


def test_unrounded_oracle_matches_autograd_mean_and_sum():
    widths = [24, 32, 16, 8, 1]
    Ws, bs = _net(1, widths)
    pooled, dense, y = _data(2, 40, 16, 8)
    for mean in (True, False):
        net = M.MLP(Ws, bs, lr=0.0, loss_mean=mean, rounding=False)
        loss, d_pooled, grads = net.step(pooled, dense, y, update=False)
        rl, rdp, rdW, rdb, _, _ = _torch_ref(Ws, bs, pooled, dense, y, mean)
        assert abs(loss - rl) < 1e-12 * max(1, abs(rl))
        np.testing.assert_allclose(d_pooled, rdp, rtol=2e-7, atol=1e-12)     # d_pooled is returned in fp32
        for (dW, db), w, b in zip(grads, rdW, rdb):
            np.testing.assert_allclose(dW, w, rtol=1e-11, atol=1e-14)
            np.testing.assert_allclose(db, b, rtol=1e-11, atol=1e-14)


def test_update_is_sgd_on_fp32_master_weights():
    widths = [12, 16, 8, 1]
    Ws, bs = _net(3, widths)
    pooled, dense, y = _data(4, 32, 8, 4)
    net = M.MLP(Ws, bs, lr=0.05, rounding=False)
    net.step(pooled, dense, y)
    _, _, _, _, tW, tb = _torch_ref(Ws, bs, pooled, dense, y, True)
    opt = torch.optim.SGD(tW + tb, lr=float(np.float32(0.05)))
    opt.step()
    for l in range(3):
        np.testing.assert_allclose(net.W[l], tW[l].detach().numpy(), rtol=2e-7, atol=1e-9)
        np.testing.assert_allclose(net.b[l], tb[l].detach().numpy(), rtol=2e-7, atol=1e-9)


def test_finite_difference_of_the_loss():
    widths = [6, 8, 4, 1]
    Ws, bs = _net(5, widths)
    pooled, dense, y = _data(6, 10, 4, 2)
    net = M.MLP(Ws, bs, lr=0.0, rounding=False)
    loss0, d_pooled, grads = net.step(pooled, dense, y, update=False)
    eps = 1e-6
    for (bb, j) in [(0, 0), (3, 2), (9, 3)]:
        p2 = pooled.astype(np.float64).copy()
        p2[bb, j] += eps
        net2 = M.MLP(Ws, bs, lr=0.0, rounding=False)
        net2.q = lambda x: np.asarray(x, dtype=np.float64)
        h = np.concatenate([p2, dense.astype(np.float64)], axis=1)
        for l in range(2):
            h = np.maximum(h @ Ws[l].astype(np.float64) + bs[l], 0)
        z = (h @ Ws[2].astype(np.float64) + bs[2]).reshape(-1)
        loss1 = np.mean(np.logaddexp(0, z) - y * z)
        assert abs((loss1 - loss0) / eps - d_pooled[bb, j]) < 1e-5 * max(1e-3, abs(d_pooled[bb, j])) + 1e-7


def test_bf16_operands_change_results_by_bf16_sized_amounts_only():
    widths = [64, 128, 64, 32, 1]
    Ws, bs = _net(7, widths)
    pooled, dense, y = _data(8, 256, 48, 16)
    exact = M.MLP(Ws, bs, lr=0.0, rounding=False).step(pooled, dense, y, update=False)
    rounded = M.MLP(Ws, bs, lr=0.0, rounding=True).step(pooled, dense, y, update=False)
    assert abs(rounded[0] - exact[0]) < 2e-2 * abs(exact[0])
    rel = np.linalg.norm(rounded[1].astype(np.float64) - exact[1]) / np.linalg.norm(exact[1])
    assert 0 < rel < 0.15, rel                                           # applied, and of bf16 size (2^-8 per operand)
    for (dWr, _), (dWe, _) in zip(rounded[2], exact[2]):
        assert np.linalg.norm(dWr - dWe) / np.linalg.norm(dWe) < 0.15
    x = np.array([1.0, 1.00390625, 1.005859375, -3.1415926, 1e-40, 65280.0], np.float32)
    np.testing.assert_array_equal(M.bf16(x), torch.tensor(x).to(torch.bfloat16).double().numpy())


def test_delayed_updates_against_autograd_on_explicitly_stale_weights():
    """delay d: the weights used at step t are w0 minus lr times the gradients of steps 0 .. t-d-1, each of
    which was itself computed on its own stale weights.  Rebuilt here step by step with torch autograd on
    explicit weight lists, for d = 2."""
    widths = [12, 16, 8, 1]
    Ws, bs = _net(3, widths)
    data = [_data(10 + t, 24, 8, 4) for t in range(5)]
    lr, d = 0.3, 2
    m = M.MLP(Ws, bs, lr=lr, loss_mean=True, rounding=False, delay=d)
    got_losses = [m.step(*data[t])[0] for t in range(5)]
    # reference: weights_at[t] = weights seen by step t
    gW, gb, want_losses = [], [], []
    for t in range(5):
        Wt = [w.astype(np.float64) for w in Ws]
        bt = [b.astype(np.float64) for b in bs]
        for k in range(max(0, t - d)):         # gradients of steps 0 .. t-d-1 have been applied, in order, in fp32
            Wt = [(w - lr * g).astype(np.float32).astype(np.float64) for w, g in zip(Wt, gW[k])]
            bt = [(b - lr * g).astype(np.float32).astype(np.float64) for b, g in zip(bt, gb[k])]
        loss, _, dWs, dbs, _, _ = _torch_ref(Wt, bt, *data[t], True)
        want_losses.append(loss)
        gW.append(dWs)
        gb.append(dbs)
    np.testing.assert_allclose(got_losses, want_losses, rtol=1e-7)   # the step size is stored as fp32 in the oracle
    assert abs(got_losses[2] - M.MLP(Ws, bs, lr=lr, rounding=False).step(*data[2])[0]) < 1e-12   # step d still sees w0
    # the weights the oracle ends with: those step 4 saw (gradients 0 .. 4-d-1 applied)
    Wend = [w.astype(np.float64) for w in Ws]
    for k in range(4 - d):
        Wend = [(w - lr * g).astype(np.float32).astype(np.float64) for w, g in zip(Wend, gW[k])]
    for w, ref in zip(m.W, Wend):
        np.testing.assert_allclose(w, ref, rtol=1e-6, atol=1e-7)


def test_zero_delay_is_the_plain_step_and_a_long_delay_changes_nothing():
    widths = [12, 16, 1]
    Ws, bs = _net(4, widths)
    data = [_data(20 + t, 16, 8, 4) for t in range(3)]
    a, b = M.MLP(Ws, bs, lr=0.2, rounding=False), M.MLP(Ws, bs, lr=0.2, rounding=False, delay=0)
    for t in range(3):
        assert a.step(*data[t])[0] == b.step(*data[t])[0]
    c = M.MLP(Ws, bs, lr=0.2, rounding=False, delay=7)
    for t in range(3):
        c.step(*data[t])
    for w, w0 in zip(c.W, Ws):
        np.testing.assert_array_equal(w, w0)
