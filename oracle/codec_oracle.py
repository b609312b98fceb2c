"""CPU oracle of the lossy value codec -- TEST INFRASTRUCTURE (numpy only).

Section 4.2.3, "Lossy compression": each fp32 vector block v is scaled by kappa / ||v||_inf and
converted to fp16; the receiver converts back to fp32 and divides by the same factor.  The paper
fixes the precisions (fp32 in, fp16 on the wire, fp32 out), so the steps below are taken in exactly
those types, in the paper's order.  Readings where the paper is silent: a block is a run of
`block_len` consecutive values; the factor is computed once per block in fp32 from the transmitted
norm; fp32 -> fp16 rounds to nearest even; a block of zeros is sent as zeros with factor 0.
"""
import numpy as np


def compress(v, block_len, kappa):
    """v: fp32 [n_blocks * block_len] -> (q fp16 [n_blocks, block_len], norm fp32 [n_blocks])."""
    v = np.ascontiguousarray(v, dtype=np.float32).reshape(-1, block_len)
    norm = np.abs(v).max(axis=1).astype(np.float32)                  # ||v||_inf per block
    with np.errstate(divide="ignore"):
        factor = np.where(norm > 0, np.float32(kappa) / norm, np.float32(0)).astype(np.float32)
    q = (v * factor[:, None]).astype(np.float32).astype(np.float16)  # scale in fp32, then convert
    return q, norm


def decompress(q, norm, kappa):
    """(q fp16 [n_blocks, block_len], norm fp32 [n_blocks]) -> fp32 [n_blocks, block_len]."""
    norm = np.asarray(norm, dtype=np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        factor = np.where(norm > 0, np.float32(kappa) / norm, np.float32(1)).astype(np.float32)
        out = q.astype(np.float32) / factor[:, None]                 # convert back, divide by the same factor
    return np.where(norm[:, None] > 0, out, np.float32(0)).astype(np.float32)
