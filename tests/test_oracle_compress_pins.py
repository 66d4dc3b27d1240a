"""Pins of the oracle's parameter-free visual token compressors (SpecVLM Sec. 3.4: the pruning
expert discards a random subset of the tokens, pooling is a plain operator; Table 4: ratios 2x to 30x).  Both are plain
definitions; they are pinned against numpy's reshape-mean / fancy indexing and closed forms."""
import numpy as np
import pytest

import workloads as W


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("T,ratio", [(576, 2), (576, 3), (577, 5), (2880, 20), (100, 30), (7, 10)])
def test_pool_against_numpy(oracle, dtype, T, ratio):
    rng = np.random.default_rng(T + ratio)
    B, E = 2, 24
    x = W.normal(rng, (B, T, E), 1.0, dtype)
    y, nt = oracle.visual_pool(x, ratio)
    xf = W.as_f64(x)
    full = T // ratio
    want = xf[:, :full * ratio].reshape(B, full, ratio, E).mean(axis=2)
    np.testing.assert_allclose(y[:, :full], want, rtol=0, atol=1e-13)
    Tp = -(-T // ratio)
    assert y.shape[1] == Tp and np.all(nt == Tp)
    if T % ratio:
        np.testing.assert_allclose(y[:, full], xf[:, full * ratio:].mean(axis=1), rtol=0, atol=1e-13)


def test_pool_closed_forms_and_ragged_lengths(oracle):
    rng = np.random.default_rng(1)
    x = rng.normal(size=(3, 50, 8)).astype(np.float32)
    y1, _ = oracle.visual_pool(x, 1)                                      # ratio 1: identity
    assert np.array_equal(y1, x.astype(np.float64))
    c = np.full((1, 33, 4), 2.5, dtype=np.float32)                        # constant stays constant, tail included
    yc, _ = oracle.visual_pool(c, 4)
    assert np.all(yc == 2.5) and yc.shape[1] == 9
    ramp = np.arange(20, dtype=np.float32).reshape(1, 20, 1)              # mean of t0..t0+r-1 is t0 + (r-1)/2
    yr, _ = oracle.visual_pool(ramp, 5)
    assert yr[0, :, 0].tolist() == [2.0, 7.0, 12.0, 17.0]
    a, b = rng.normal(size=(2, 1, 40, 6)).astype(np.float32)              # linearity of the mean
    ya, yb = oracle.visual_pool(a, 3)[0], oracle.visual_pool(b, 3)[0]
    yab = oracle.visual_pool((a.astype(np.float64) * 2 + b).astype(np.float32), 3)[0]
    np.testing.assert_allclose(yab, 2 * ya + yb, atol=1e-5)
    nt = np.array([50, 17, 0], dtype=np.int32)                            # per-request lengths
    y, out = oracle.visual_pool(x, 4, nt)
    assert out.tolist() == [13, 5, 0]
    np.testing.assert_allclose(y[1, 4], x[1, 16:17].astype(np.float64).mean(axis=0), atol=1e-15)
    assert np.all(y[1, 5:] == 0) and np.all(y[2] == 0)
    with pytest.raises(ValueError):
        oracle.visual_pool(x, 4, np.array([51, 0, 0]))


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_prune_against_fancy_indexing(oracle, dtype):
    rng = np.random.default_rng(2)
    B, T, E, keep_n = 3, 576, 40, 29                                      # 576 / 20 rounded up
    x = W.normal(rng, (B, T, E), 1.0, dtype)
    keep = np.stack([np.sort(rng.choice(T, keep_n, replace=False)) for _ in range(B)]).astype(np.int32)
    keep[2, -5:] = -1                                                     # padding rows
    keep[1, :3] = [575, 0, 575]                                           # any order, repeats
    y = oracle.visual_prune(x, keep)
    for b in range(B):
        real = keep[b] >= 0
        assert np.array_equal(y[b, real], x[b, keep[b, real]])
        assert np.all(y[b, ~real] == 0)
    big = W.normal(rng, (B, T, 3 * E), 1.0, dtype)                        # features inside a wider buffer
    assert np.array_equal(oracle.visual_prune(big[:, :, E:2 * E], keep)[0, :5], big[0, keep[0, :5], E:2 * E])
    with pytest.raises(ValueError):
        oracle.visual_prune(x, np.full((B, 2), T, dtype=np.int32))
