"""GPU parity of the optional dense step (Algorithm 2 on one GPU) against its fp64 oracle, and of the bf16
MFMA contraction it is built from against a plain matrix product.  Tolerance for everything that passed
through bf16 operands: 2e-2 relative (the benchmark spec), with an absolute floor tied to the scale of the tensor."""
import numpy as np
import pytest

from oracle import mlp_oracle as MO

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2111_05897_amd import binding
    binding.load_library()
    return binding


def _close(got, want, rtol=2e-2, floor=2e-3):
    want = np.asarray(want, dtype=np.float64)
    scale = np.abs(want).max() if want.size else 0.0
    np.testing.assert_allclose(got, want, rtol=rtol, atol=floor * scale)


@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (64, 32, 128), (300, 200, 192), (129, 257, 64), (1, 1, 64),
                                   (512, 9920 // 8, 256), (700, 520, 128), (257, 1033, 64)])
def test_gemm_nt_matches_fp64_product(B, M, N, K):
    import torch
    rng = np.random.default_rng(M * 7 + N)
    A = torch.tensor(rng.standard_normal((M, K)), dtype=torch.bfloat16)
    Bt = torch.tensor(rng.standard_normal((N, K)), dtype=torch.bfloat16)
    want = A.double().numpy() @ Bt.double().numpy().T
    got = B.mlp_gemm_nt(1, A.cuda(), Bt.cuda()).cpu().numpy()
    # fp32 accumulation of exact bf16 products: error ~ K * 2^-24 relative to the magnitude of the terms
    np.testing.assert_allclose(got, want, rtol=1e-4, atol=1e-4 * np.sqrt(K))
    bias = torch.tensor(rng.standard_normal(N), dtype=torch.float32)
    got0 = B.mlp_gemm_nt(0, A.cuda(), Bt.cuda(), bias=bias.cuda()).float().cpu().numpy()
    want0 = torch.tensor(np.maximum(want + bias.double().numpy(), 0)).to(torch.bfloat16).float().numpy()
    _close(got0, want0, rtol=8e-3, floor=1e-3)              # one bf16 rounding apart at most
    mask = torch.tensor(rng.standard_normal((M, N)), dtype=torch.bfloat16)
    got2 = B.mlp_gemm_nt(2, A.cuda(), Bt.cuda(), mask=mask.cuda()).float().cpu().numpy()
    want2 = np.where(mask.float().numpy() > 0, want, 0.0)
    _close(got2, want2, rtol=8e-3, floor=1e-3)
    assert (got2[mask.float().numpy() <= 0] == 0).all()


def test_gemm_nt_rejects_bad_shapes(B):
    import torch
    A = torch.zeros((64, 100), dtype=torch.bfloat16, device="cuda")       # K not a multiple of 64
    with pytest.raises(B.EmbError):
        B.mlp_gemm_nt(1, A, A)


def _net(seed, widths):
    rng = np.random.default_rng(seed)
    Ws = [(rng.standard_normal((i, o)) * np.sqrt(2.0 / i)).astype(np.float32) for i, o in zip(widths[:-1], widths[1:])]
    bs = [(rng.standard_normal(o) * 0.05).astype(np.float32) for o in widths[1:]]
    return Ws, bs


@pytest.mark.parametrize("widths,P,Bsz,mean", [([128, 256, 128, 64, 1], 64, 256, True),
                                               ([192, 128, 64, 1], 128, 320, False),
                                               ([1024 + 64, 512, 256, 128, 1], 1024, 1024, True)])
def test_mlp_step_matches_oracle_stage_by_stage(B, widths, P, Bsz, mean):
    """Every stage of the step is compared with the oracle's stage function applied to the GPU's own stage
    inputs (read back with mlp_read_state), so a ReLU that falls on the other side of zero for one sample --
    a legitimate outcome when a pre-activation is within rounding of zero -- cannot masquerade as, or hide, an
    arithmetic error further down.  The whole step is then compared with the oracle's whole step in norm."""
    import torch
    Dn = widths[0] - P
    L = len(widths) - 1
    Ws, bs = _net(len(widths) + P, widths)
    lr = 0.05
    ctx = B.MlpContext(widths, P, Dn, Bsz, lr, Ws, bs, loss_mean=mean)
    orc = MO.MLP(Ws, bs, lr=lr, loss_mean=mean, rounding=True)
    q = orc.q
    rng = np.random.default_rng(3)
    ULP = 2.0 ** -7                                   # one bf16 rounding apart at most
    for step in range(2):
        W_before = [w.copy() for w in orc.W]
        b_before = [b.copy() for b in orc.b]
        pooled = (rng.standard_normal((Bsz, P)) * 0.2).astype(np.float32)
        dense = rng.standard_normal((Bsz, Dn)).astype(np.float32)
        y = (rng.random(Bsz) < 0.05).astype(np.float32)
        d_pooled, loss = ctx.mlp_step(torch.from_numpy(pooled).cuda(), torch.from_numpy(dense).cuda(),
                                      torch.from_numpy(y).cuda())
        torch.cuda.synchronize()
        d_pooled = d_pooled.cpu().numpy()
        h = [ctx.mlp_read_state("h", l, Bsz).astype(np.float64) for l in range(L)]
        delta = [None] + [ctx.mlp_read_state("delta", l, Bsz).astype(np.float64) for l in range(1, L)]
        # forward
        np.testing.assert_array_equal(h[0], q(np.concatenate([pooled, dense], axis=1)))
        for l in range(L - 1):
            ref, a = MO.layer_forward(h[l], W_before[l], b_before[l], q)
            np.testing.assert_allclose(h[l + 1], ref, rtol=ULP, atol=1e-5 + 1e-6 * np.abs(a).max())
        scale = 1.0 / Bsz if mean else 1.0
        _, ref_loss, ref_dz = MO.logit_loss(h[L - 1], q(W_before[L - 1]), b_before[L - 1], y.astype(np.float64), scale)
        assert abs(loss.item() - ref_loss) <= 1e-5 * abs(ref_loss)
        dz = ctx.mlp_read_state("dz", 0, Bsz).astype(np.float64)
        np.testing.assert_allclose(dz, ref_dz, rtol=1e-4, atol=1e-7 * scale)
        # backward
        np.testing.assert_allclose(delta[L - 1], MO.delta_from_logit(dz, q(W_before[L - 1]), h[L - 1], q), rtol=ULP,
                                   atol=1e-12)
        for l in range(L - 1, 0, -1):
            dW_ref, db_ref = MO.weight_grad(h[l - 1], delta[l])
            _close(ctx.mlp_read_state("dW", l - 1, Bsz), dW_ref, rtol=1e-3, floor=1e-4)
            _close(ctx.mlp_read_state("db", l - 1, Bsz), db_ref, rtol=1e-3, floor=1e-4)
            if l >= 2:
                _close(delta[l - 1], MO.delta_back(delta[l], W_before[l - 1], h[l - 1], q), rtol=ULP, floor=1e-4)
        _close(ctx.mlp_read_state("dW", L - 1, Bsz).reshape(-1), (h[L - 1].T @ dz[:, None]).reshape(-1), rtol=1e-3, floor=1e-4)
        _close(ctx.mlp_read_state("db", L - 1, Bsz), np.array([dz.sum()]), rtol=1e-3, floor=1e-4)
        _close(d_pooled, (delta[1] @ q(W_before[0]).T)[:, :P], rtol=1e-3, floor=1e-4)
        # update: plain SGD on the fp32 master weights with the GPU's own gradients
        for l in range(L):
            gw, gb = ctx.mlp_read_weights(l)
            want_w = (W_before[l].astype(np.float64) - float(np.float32(lr)) * ctx.mlp_read_state("dW", l, Bsz)).astype(np.float32)
            np.testing.assert_allclose(gw, want_w, rtol=3e-7, atol=1e-7 * np.abs(want_w).max())   # one fp32 rounding
            want_b = (b_before[l].astype(np.float64) - float(np.float32(lr)) * ctx.mlp_read_state("db", l, Bsz)).astype(np.float32)
            np.testing.assert_allclose(gb, want_b, rtol=3e-7, atol=1e-7 * max(np.abs(want_b).max(), 1e-30))
        # whole step against the oracle's whole step, in norm (individual samples may differ by a ReLU decision)
        oloss, odp, _ = orc.step(pooled, dense, y)
        assert abs(loss.item() - oloss) <= 2e-2 * abs(oloss)
        assert np.linalg.norm(d_pooled - odp) <= 2e-2 * np.linalg.norm(odp)
        for l in range(L):   # keep both sides on one trajectory: continue from the GPU's weights
            orc.W[l], orc.b[l] = ctx.mlp_read_weights(l)
    assert ctx.mlp_device_bytes() > 0
    ctx.close()


def test_mlp_create_rejects_bad_configurations(B):
    Ws, bs = _net(1, [100, 64, 1])
    with pytest.raises(B.EmbError):
        B.MlpContext([100, 64, 1], 36, 64, 64, 0.1, Ws, bs)               # input width not a multiple of 64
    Ws, bs = _net(1, [128, 64, 2])
    with pytest.raises(B.EmbError):
        B.MlpContext([128, 64, 2], 64, 64, 64, 0.1, Ws, bs)               # two outputs


def test_delayed_updates_follow_the_oracle(B):
    """mlp_set_update_delay: step t works with weights that miss the gradients of the last d steps.  Losses and
    the movement of the weights against the oracle with the same delay; a delay beyond the run leaves the
    weights bit-identical; a context cannot change its delay after a step."""
    import torch
    widths, P, Bsz, d = [128 + 64, 256, 128, 1], 128, 256, 2
    Dn = widths[0] - P
    Ws, bs = _net(9, widths)
    ctx = B.MlpContext(widths, P, Dn, Bsz, 0.1, Ws, bs, loss_mean=True)
    ctx.mlp_set_update_delay(d)
    orc = MO.MLP(Ws, bs, lr=0.1, loss_mean=True, rounding=True, delay=d)
    frozen = B.MlpContext(widths, P, Dn, Bsz, 0.1, Ws, bs, loss_mean=True)
    frozen.mlp_set_update_delay(50)
    rng = np.random.default_rng(5)
    got, want = [], []
    for t in range(7):
        pooled = (rng.standard_normal((Bsz, P)) * 0.3).astype(np.float32)
        dense = rng.standard_normal((Bsz, Dn)).astype(np.float32)
        y = (rng.random(Bsz) < 0.3).astype(np.float32)
        args = (torch.from_numpy(pooled).cuda(), torch.from_numpy(dense).cuda(), torch.from_numpy(y).cuda())
        got.append(ctx.mlp_step(*args)[1].item())
        frozen.mlp_step(*args)
        want.append(orc.step(pooled, dense, y)[0])
    np.testing.assert_allclose(got, want, rtol=2e-2)
    for l in range(len(widths) - 1):
        gw, gb = ctx.mlp_read_weights(l)
        moved = np.linalg.norm(orc.W[l].astype(np.float64) - Ws[l])
        assert moved > 0 and np.linalg.norm(gw - orc.W[l]) <= 3e-2 * moved
        fw, fb = frozen.mlp_read_weights(l)
        np.testing.assert_array_equal(fw, Ws[l])
        np.testing.assert_array_equal(fb, bs[l])
    with pytest.raises(B.EmbError):
        ctx.mlp_set_update_delay(1)
