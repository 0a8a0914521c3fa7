"""Test helpers: move encoded operands between the GPU library's stored layout and the
source-orientation arrays the oracle works on.  Pure index shuffling, no arithmetic."""
import os

import numpy as np


def random_cases(default):
    """Seeds of a randomised test: `default` of them, or HBFP_RANDOM_CASES if set (a longer soak of the same test)."""
    return range(int(os.environ.get("HBFP_RANDOM_CASES", default)))


def unpack(bt):
    """BfpTensor (GPU, operand layout) -> (mant int32 [src_rows, src_cols], exps uint8 [nbr, nbc]).

    Also asserts what the layout promises: zero padding, exponent padding bytes of 1, and equal
    exponent bytes on operand rows that share a 2-D block."""
    d = bt.desc
    mant = bt.mant.cpu().numpy().astype(np.int32)
    exps = bt.exps.cpu().numpy()
    R, K, kb, kbp, nblk = d.rows, d.kdim, d.kblock, d.kblock_pad, d.nblk
    assert mant.shape == (R, d.kpad) and exps.shape == (R, d.exp_ld)
    nst = d.kpad // kbp
    blocks = mant.reshape(R, nst, kbp)
    assert (blocks[:, nblk:, :] == 0).all(), "padding blocks must be zero"
    assert (blocks[:, :, kb:] == 0).all(), "padding inside blocks must be zero"
    op = blocks[:, :nblk, :kb].reshape(R, nblk * kb)
    assert (op[:, K:] == 0).all(), "tail of the last block must be zero"
    op = op[:, :K]
    assert (exps[:, nblk:] == 1).all(), "exponent padding must be 1"
    e = exps[:, :nblk]
    ks = min(d.kshare, nblk)
    assert (np.repeat(e[:, ::ks], ks, axis=1)[:, :nblk] == e).all(), "stored blocks of one exponent block must repeat the exponent"
    e = e[:, ::ks]
    rb = d.rblock
    first = e[::rb]
    assert (np.repeat(first, rb, axis=0)[:R] == e).all(), "rows of one 2-D block must repeat the exponent"
    if d.contract_axis == 1:
        return np.ascontiguousarray(op), np.ascontiguousarray(first)
    return np.ascontiguousarray(op.T), np.ascontiguousarray(first.T)


def rel_fro(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))
