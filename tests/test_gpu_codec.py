"""GPU parity of the scaled-fp16 value codec (section 4.2.3, lossy compression) against its numpy oracle.
Both sides do the same fp32 operations and the same fp32->fp16 rounding, so codes, norms and the
decompressed values are compared bit for bit."""
import numpy as np
import pytest

from oracle import codec_oracle as CO

pytestmark = pytest.mark.gpu
KAPPA = 2.0 ** 15


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2111_05897_amd import binding
    binding.load_library()
    return binding


@pytest.mark.parametrize("n_blocks,block_len,scale", [(1, 4, 1.0), (7, 8, 1e-4), (1000, 64, 1.0), (333, 100, 50.0),
                                                       (129, 1028, 1e-12), (64, 3200, 1.0), (17, 9920, 0.01),
                                                       (3, 20000, 1e8), (0, 64, 1.0)])
def test_codec_matches_oracle_bit_exact(B, n_blocks, block_len, scale):
    import torch
    rng = np.random.default_rng(n_blocks * 131 + block_len)
    v = (rng.standard_normal((n_blocks, block_len)) * scale).astype(np.float32)
    if n_blocks > 2:
        v[1] = 0.0                                   # a block of zeros
        v[2, 1:] *= np.float32(1e-7)                 # one dominant element: the rest lands in fp16's subnormals
    dv = torch.from_numpy(v).cuda()
    q, norm = B.emb_codec_compress(dv, block_len, KAPPA)
    out = B.emb_codec_decompress(q, norm, KAPPA)
    torch.cuda.synchronize()
    if n_blocks == 0:
        assert q.shape == (0, block_len)
        return
    oq, onorm = CO.compress(v, block_len, KAPPA)
    np.testing.assert_array_equal(norm.cpu().numpy(), onorm)
    np.testing.assert_array_equal(q.cpu().numpy().view(np.uint16), oq.view(np.uint16))
    np.testing.assert_array_equal(out.cpu().numpy().view(np.uint32), CO.decompress(oq, onorm, KAPPA).view(np.uint32))
    # and the paper's point: the round trip stays within 2^-11 of the block norm
    assert (np.abs(out.cpu().numpy().astype(np.float64) - v) <= onorm[:, None] * 2.0 ** -11 * (1 + 1e-6)).all()


def test_codec_on_pooled_activations_of_config2_shape(B):
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    v = torch.randn((2048, 6400), generator=gen, device="cuda", dtype=torch.float32) * 0.05
    for block_len in (64, 6400):                     # one slot's vector / one sample's pooled row
        q, norm = B.emb_codec_compress(v, block_len, KAPPA)
        out = B.emb_codec_decompress(q, norm, KAPPA)
        torch.cuda.synchronize()
        hv = v.cpu().numpy()
        oq, onorm = CO.compress(hv, block_len, KAPPA)
        np.testing.assert_array_equal(q.cpu().numpy().view(np.uint16), oq.view(np.uint16))
        np.testing.assert_array_equal(out.cpu().numpy(), CO.decompress(oq, onorm, KAPPA))


def test_codec_rejects_bad_arguments(B):
    import torch
    v = torch.zeros(64, device="cuda")
    with pytest.raises(B.EmbError):
        B.emb_codec_compress(v, 64, 1e6)             # kappa beyond fp16's largest finite value
    with pytest.raises(B.EmbError):
        B.emb_codec_compress(torch.zeros(66, device="cuda"), 6, KAPPA)   # block_len not a multiple of 4
