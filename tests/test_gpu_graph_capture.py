"""The hot calls only enqueue kernels on the caller's stream, so a whole step (lookup + backward/update) can be
captured in a HIP graph and replayed.  The test captures one step, replays it several times with unrelated eager
work and synchronisations in between, and checks every replay bit for bit against the same calls enqueued
directly on a second context: pooled activations after each step, the index form, and every row at the end."""
import numpy as np
import pytest

from paper_2111_05897_amd import workload as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2111_05897_amd import binding
    binding.load_library()
    return binding


@pytest.mark.parametrize("tables,slots,opt", [([(1 << 12, 64, 0)], [0] * 6, 1),
                                               ([(3000, 16, 1), (1 << 10, 128, 0)], [0, 1, 1, 0, 0], 0)])
def test_captured_step_replays_like_direct_calls(B, tables, slots, opt):
    import torch
    S, bsz = len(slots), 96
    args = dict(tables=tables, slots=[(t, W.default_salt(s)) for s, t in enumerate(slots)], hash_kind=1, opt=opt,
                lr=0.05, eps=1e-8, acc_init=0.1, init_seed=77, init_lo=-0.05, init_hi=0.05)
    b = W.random_batch(4242, bsz, S, 9, 700)
    direct = B.EmbContext(max_batch=bsz, max_ids=b.num_ids, **args)
    graphed = B.EmbContext(max_batch=bsz, max_ids=b.num_ids, **args)
    db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
    width = sum(tables[t][1] for t in slots)
    dp = torch.from_numpy(np.random.default_rng(3).standard_normal((bsz, width)).astype(np.float32)).cuda()
    pooled_d = torch.empty((bsz, width), dtype=torch.float32, device="cuda")
    pooled_g = torch.full((bsz, width), float("nan"), dtype=torch.float32, device="cuda")

    side = torch.cuda.Stream()                       # default priority
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):   # nothing runs here: the calls are recorded
            graphed.emb_lookup_pool(db, pooled_g)
            graphed.emb_backward_update(db, dp)
    torch.cuda.synchronize()

    for step in range(4):
        direct.emb_lookup_pool(db, pooled_d)
        direct.emb_backward_update(db, dp)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(pooled_g, pooled_d), f"pooled differs at replay {step}"
        for x, y in zip(graphed.emb_read_dedup(), direct.emb_read_dedup()):
            np.testing.assert_array_equal(x, y)
        # the program's own eager work between replays
        junk = torch.randn(1 << 16, device="cuda").cumsum(0)
        pooled_g.fill_(float("nan"))
        torch.cuda.synchronize()
        del junk
    for t, (rows, _, _) in enumerate(tables):
        gw, ga = graphed.emb_read_rows(t, np.arange(rows))
        dw, da = direct.emb_read_rows(t, np.arange(rows))
        np.testing.assert_array_equal(gw, dw)
        np.testing.assert_array_equal(ga, da)
    del graph
    graphed.close()
    direct.close()


def test_captured_dense_step_replays_like_direct_calls(B):
    """mlp_step (forward, loss, backward, SGD step: a few dozen kernels, split-K workspaces included) captured once
    and replayed three times against the same call enqueued directly: gradients of the pooled activations, losses
    and the updated weights, bit for bit."""
    import torch
    P, Dn, bsz = 192, 64, 256
    widths = [P + Dn, 256, 128, 1]
    Ws, bs = W.make_mlp_params(widths, 5)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    pooled = torch.randn((bsz, P), generator=gen, device="cuda")
    dense = torch.randn((bsz, Dn), generator=gen, device="cuda")
    labels = (torch.rand((bsz,), generator=gen, device="cuda") < 0.3).float()
    out = {}
    for mode in ("direct", "graph"):
        mlp = B.MlpContext(widths, P, Dn, bsz, 0.1, Ws, bs, loss_mean=True)
        d_pooled = torch.empty_like(pooled)
        if mode == "graph":
            side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    _, loss = mlp.mlp_step(pooled, dense, labels, d_pooled)
            torch.cuda.synchronize()
        seen = []
        for _ in range(3):
            if mode == "graph":
                graph.replay()
            else:
                _, loss = mlp.mlp_step(pooled, dense, labels, d_pooled)
            torch.cuda.synchronize()
            seen.append((d_pooled.clone(), loss.clone()))
            d_pooled.fill_(float("nan"))
            torch.randn(1 << 16, device="cuda").sum().item()     # eager work between the replays
        out[mode] = (seen, [mlp.mlp_read_weights(l) for l in range(len(widths) - 1)])
        if mode == "graph":
            del graph
        mlp.close()
    for (dp_d, loss_d), (dp_g, loss_g) in zip(out["direct"][0], out["graph"][0]):
        assert torch.equal(dp_d, dp_g) and torch.equal(loss_d, loss_g)
    for (w_d, b_d), (w_g, b_g) in zip(out["direct"][1], out["graph"][1]):
        np.testing.assert_array_equal(w_d, w_g)
        np.testing.assert_array_equal(b_d, b_g)
