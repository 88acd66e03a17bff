"""The reason the paper gives for tensor chunking (Sec. IV-B): independent per-block
normalization keeps outliers from destroying the precision of the other blocks.  Checked on
the oracle: with outliers, the round-trip error of block-wise quantization falls as B
shrinks and is far below whole-tensor quantization; the absmax overhead is 4/B bytes per
state entry."""
import numpy as np

import oracle

QS = oracle.build_codebook(True)


def roundtrip_rel_rms(T, B):
    TQ, N = oracle.quantize_blockwise(QS, T, B)
    TD = oracle.dequantize_blockwise(QS, TQ, N, B)
    return float(np.sqrt(np.mean((TD.astype(np.float64) - T) ** 2)) / np.sqrt(np.mean(T.astype(np.float64) ** 2)))


def test_smaller_blocks_contain_outliers():
    rng = np.random.default_rng(0)
    n = 1 << 18
    T = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    clean = {B: roundtrip_rel_rms(T, B) for B in (256, 2048, n)}
    # without outliers the block size hardly matters
    assert abs(clean[256] - clean[2048]) < 0.5 * clean[2048]
    for mult, whole_vs_2048 in ((1e3, 1.5), (1e5, 1.7), (1e7, 1.8)):
        out = T.copy()
        idx = rng.choice(n, n // 4096, replace=False)              # one outlier per 4096 entries
        out[idx] *= mult
        mask = np.ones(n, bool); mask[idx] = False                  # error on the ordinary entries only

        def err(B):
            TQ, N = oracle.quantize_blockwise(QS, out, B)
            TD = oracle.dequantize_blockwise(QS, TQ, N, B)
            d = (TD.astype(np.float64) - out)[mask]
            return float(np.sqrt(np.mean(d ** 2)) / np.sqrt(np.mean(out[mask].astype(np.float64) ** 2)))

        e = {B: err(B) for B in (64, 256, 2048, 4096, n)}
        assert e[64] < e[256] < e[2048] < e[4096] < e[n], (mult, e)
        assert e[n] > whole_vs_2048 * e[2048] and e[2048] > 2 * e[256], (mult, e)
    # an outlier 10^7 times the typical entry wipes out a whole-tensor quantization
    # (every ordinary entry rounds to zero) but only its own block when B is small
    assert e[n] > 0.99 and e[64] < 0.11


def test_absmax_overhead_per_block_size():
    for B in (64, 256, 2048, 4096):
        n = 10 * B + 1
        TQ, N = oracle.quantize_blockwise(QS, np.ones(n, np.float32), B)
        assert TQ.nbytes == n and N.nbytes == 4 * 11
