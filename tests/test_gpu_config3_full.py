"""Configuration 3 as BASELINE names it, at full size, in one chained step: lookup over 200 slots of five bf16 tables
(2^27 rows in all, 108 M ids) -> dense step of the network 10432-4096-2048-1024-1 at batch 32768 (Algorithm 2: bf16
MFMA contractions, among them the K = 32768 weight-gradient products that are cut along K) -> embedding update fed
with the network's own gradient of the pooled activations (Algorithm 1, backward task).

What is compared, stage by stage (each stage against the oracle's definition applied to the GPU's own stage inputs,
so that bf16 noise of one stage never passes for -- or hides -- an error of the next):
  * pooled activations of sampled bags, the whole index form, updated rows / accumulators / bag lists of sampled
    unique rows: tests/util.sampled_step_check with the dense step in the middle;
  * every large contraction of the dense step on sampled output elements, against fp64 dot products of the GPU's
    own bf16 operands (read back with mlp_read_state), the logit / loss / dz and the last hidden delta in full,
    and the SGD update of sampled weights."""
import numpy as np
import pytest

from oracle import mlp_oracle as MO
from oracle import oracle as O
from paper_2111_05897_amd import workload as W
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2111_05897_amd import binding
    binding.load_library()
    return binding


STATE = {}


def test_chained_step_embedding_side(B):
    import torch
    w = W.make_workload(3)
    P = w.cfg.pooled_width
    widths = [P + W.DENSE_FEATURES] + W.MLP_HIDDEN + [1]
    assert widths == [10432, 4096, 2048, 1024, 1] and w.batch == 32768
    Ws, bs = W.make_mlp_params(widths, w.seed)
    lr = 1e-3
    mlp = B.MlpContext(widths, P, W.DENSE_FEATURES, w.batch, lr, Ws, bs, loss_mean=True)
    dense, y = W.make_dense_and_labels(w.seed, 0, w.batch)
    out = {}

    def dense_step(pooled_dev):
        d_pooled, loss = mlp.mlp_step(pooled_dev, torch.from_numpy(dense).cuda(), torch.from_numpy(y).cuda())
        torch.cuda.synchronize()
        out["loss"] = float(loss.item())
        out["pooled"] = pooled_dev.cpu().numpy()
        return d_pooled

    util.sampled_step_check(B, W, O, w, dense_step=dense_step)
    STATE.update(mlp=mlp, widths=widths, Ws=Ws, bs=bs, lr=lr, dense=dense, y=y, P=P, Bsz=w.batch, **out)


def _sample(rng, n, *dims):
    return [rng.integers(0, d, size=n) for d in dims]


def test_chained_step_dense_side_sampled_products():
    assert "mlp" in STATE, "the chained step did not run"
    mlp, widths, Ws, bs, lr = STATE["mlp"], STATE["widths"], STATE["Ws"], STATE["bs"], STATE["lr"]
    Bsz, P = STATE["Bsz"], STATE["P"]
    L = len(widths) - 1
    q = MO.bf16
    rng = np.random.default_rng(33)
    ULP = 2.0 ** -7
    NS = 384
    h = [mlp.mlp_read_state("h", l, Bsz) for l in range(L)]                 # bf16 values widened to fp32
    delta = [None] + [mlp.mlp_read_state("delta", l, Bsz) for l in range(1, L)]
    # packed input: [pooled | dense] rounded to bf16 (every 8th sample of the pooled part, the dense part in full)
    np.testing.assert_array_equal(h[0][::8, :P], q(STATE["pooled"][::8]).astype(np.float32))
    np.testing.assert_array_equal(h[0][:, P:], q(STATE["dense"]).astype(np.float32))
    # forward products (K = 10432, 4096, 2048)
    for l in range(L - 1):
        i, j = _sample(rng, NS, Bsz, widths[l + 1])
        a = np.einsum("nk,nk->n", h[l][i].astype(np.float64), q(Ws[l][:, j].T)) + bs[l][j]
        want = q(np.maximum(a, 0.0).astype(np.float32))
        np.testing.assert_allclose(h[l + 1][i, j], want, rtol=ULP, atol=1e-5 + 1e-6 * np.abs(a).max(), err_msg=f"forward layer {l}")
    # logit, loss, dz, last hidden delta: in full
    scale = 1.0 / Bsz
    _, ref_loss, ref_dz = MO.logit_loss(h[L - 1].astype(np.float64), q(Ws[L - 1]), bs[L - 1], STATE["y"].astype(np.float64), scale)
    assert abs(STATE["loss"] - ref_loss) <= 1e-5 * abs(ref_loss)
    dz = mlp.mlp_read_state("dz", 0, Bsz).astype(np.float64)
    np.testing.assert_allclose(dz, ref_dz, rtol=1e-4, atol=1e-7 * scale)
    np.testing.assert_allclose(delta[L - 1], MO.delta_from_logit(dz, q(Ws[L - 1]), h[L - 1].astype(np.float64), q), rtol=ULP, atol=1e-12)
    # back-propagated deltas (K = 1024, 2048), masked by the stored activation
    for l in range(L - 1, 1, -1):
        i, j = _sample(rng, NS, Bsz, widths[l - 1])
        a = np.einsum("nk,nk->n", delta[l][i].astype(np.float64), q(Ws[l - 1][j, :])) * (h[l - 1][i, j] > 0)
        scale_d = np.abs(delta[l - 1]).max()
        np.testing.assert_allclose(delta[l - 1][i, j], q(a.astype(np.float32)), rtol=ULP, atol=1e-4 * scale_d, err_msg=f"delta {l - 1}")
    # weight gradients: K = 32768 (the batch), cut along K on the GPU
    dWs = []
    for l in range(L - 1):
        dW = mlp.mlp_read_state("dW", l, Bsz)
        dWs.append(dW)
        i, j = _sample(rng, NS, widths[l], widths[l + 1])
        want = np.array([np.dot(h[l][:, a_].astype(np.float64), delta[l + 1][:, b_].astype(np.float64)) for a_, b_ in zip(i, j)])
        np.testing.assert_allclose(dW[i, j], want, rtol=1e-3, atol=1e-4 * np.abs(want).max(), err_msg=f"weight gradient {l}")
        db = mlp.mlp_read_state("db", l, Bsz)
        np.testing.assert_allclose(db, delta[l + 1].astype(np.float64).sum(axis=0), rtol=1e-3, atol=1e-4 * np.abs(db).max())
    dWs.append(mlp.mlp_read_state("dW", L - 1, Bsz))
    np.testing.assert_allclose(dWs[-1].reshape(-1), h[L - 1].astype(np.float64).T @ dz, rtol=1e-3, atol=1e-4 * np.abs(dWs[-1]).max())
    # SGD on the fp32 master weights with the GPU's own gradients, sampled
    for l in range(L):
        gw, gb = mlp.mlp_read_weights(l)
        i, j = _sample(rng, 4096, widths[l], widths[l + 1])
        want = (Ws[l][i, j].astype(np.float64) - float(np.float32(lr)) * dWs[l][i, j]).astype(np.float32)
        np.testing.assert_allclose(gw[i, j], want, rtol=3e-7, atol=1e-7 * np.abs(want).max(), err_msg=f"weights {l}")
    STATE["delta1"], STATE["h0"] = delta[1], None


def test_chained_step_gradient_of_pooled_activations(B):
    """d_pooled = delta_1 W_0^T restricted to the pooled columns (K = 4096), on sampled elements: the dense step is run
    again on the same inputs with fresh weights (the first run's d_pooled buffer was consumed by the update)."""
    import torch
    assert "delta1" in STATE
    widths, Ws, bs, P, Bsz = STATE["widths"], STATE["Ws"], STATE["bs"], STATE["P"], STATE["Bsz"]
    STATE.pop("mlp").close()
    mlp = B.MlpContext(widths, P, W.DENSE_FEATURES, Bsz, STATE["lr"], Ws, bs, loss_mean=True)
    d_pooled, _ = mlp.mlp_step(torch.from_numpy(STATE["pooled"]).cuda(), torch.from_numpy(STATE["dense"]).cuda(),
                               torch.from_numpy(STATE["y"]).cuda())
    torch.cuda.synchronize()
    delta1 = mlp.mlp_read_state("delta", 1, Bsz)
    np.testing.assert_array_equal(delta1, STATE["delta1"])          # the step is reproducible bit for bit
    rng = np.random.default_rng(34)
    i, j = _sample(rng, 2048, Bsz, P)
    got = d_pooled[torch.from_numpy(i).cuda(), torch.from_numpy(j).cuda()].cpu().numpy()
    want = np.einsum("nk,nk->n", delta1[i].astype(np.float64), MO.bf16(Ws[0][j, :]))
    np.testing.assert_allclose(got, want, rtol=1e-3, atol=1e-4 * np.abs(want).max())
    mlp.close()
    STATE.clear()
