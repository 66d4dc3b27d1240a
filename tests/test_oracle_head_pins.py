"""Pins of the oracle's fused output head + greedy choice (SpecVLM Fig. 3: the output head is
shared by target and draft; Sec. 4.1: temperature 0).  The definition is a matrix product followed
by the separately pinned argmax rule, so it is pinned against numpy's float64 matmul, against
inputs whose answer is known in closed form, and against oracle_node_argmax on stored logits
in a case where the logits are exactly representable."""
import numpy as np
import pytest

import workloads as W


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_against_numpy_matmul(oracle, dtype):
    rng = np.random.default_rng(5)
    B, N, E, V = 2, 7, 96, 333
    h = W.normal(rng, (B, N, E), 1.0, dtype)
    w = W.normal(rng, (V, E), 0.3, dtype)
    nn = np.array([7, 3], dtype=np.int32)
    amax, mx, gap, second = oracle.head_argmax(h, w, nn)
    logits = W.as_f64(h) @ W.as_f64(w).T                                  # [B,N,V], float64
    for b in range(B):
        for i in range(N):
            if i >= nn[b]:
                assert amax[b, i] == -1 and second[b, i] == -1
                continue
            order = np.lexsort((np.arange(V), -logits[b, i]))
            assert amax[b, i] == order[0] and second[b, i] == order[1]
            assert abs(mx[b, i] - logits[b, i, order[0]]) < 1e-10
            assert abs(gap[b, i] - (logits[b, i, order[0]] - logits[b, i, order[1]])) < 1e-10


def test_one_hot_head_rows_pick_the_largest_component(oracle):
    """W[v] = e_{perm[v]}: logit v is hidden component perm[v], so the answer is known without any sum."""
    rng = np.random.default_rng(6)
    E = V = 40
    perm = rng.permutation(E)
    w = np.zeros((V, E), dtype=np.float32)
    w[np.arange(V), perm] = 1.0
    h = rng.normal(size=(1, 5, E)).astype(np.float32)
    amax, mx, gap, _ = oracle.head_argmax(h, w)
    inv = np.argsort(perm)                                               # token whose row selects component e
    assert np.array_equal(amax[0], inv[np.argmax(h[0], axis=1)])
    np.testing.assert_allclose(mx[0], h[0].max(axis=1).astype(np.float64), rtol=0, atol=0)
    srt = np.sort(h[0].astype(np.float64), axis=1)
    np.testing.assert_allclose(gap[0], srt[:, -1] - srt[:, -2], rtol=0, atol=1e-15)


def test_exact_integer_case_agrees_with_argmax_of_stored_logits(oracle):
    """Small integers: every product and sum is exact in fp32, so storing the logits and calling the
    separately pinned node_argmax must give the same tokens, ties included."""
    rng = np.random.default_rng(7)
    B, N, E, V = 2, 6, 32, 500
    h = rng.integers(-3, 4, size=(B, N, E)).astype(np.float32)
    w = rng.integers(-2, 3, size=(V, E)).astype(np.float32)
    w[123] = w[7]                                                        # duplicate rows: exact ties
    w[400] = w[7]
    logits = np.einsum("bne,ve->bnv", h, w).astype(np.float32)
    amax, mx, gap, second = oracle.head_argmax(h, w)
    assert np.array_equal(amax, oracle.node_argmax(logits))
    assert np.array_equal(mx, logits.max(axis=2).astype(np.float64))
    assert (gap == 0).any() and np.all(gap >= 0)                         # integer logits tie often
    tie = gap == 0
    assert np.all(second[tie] > amax[tie])                               # the lower token wins a tie
    for bb in range(B):                                                  # runner-up: same rule among the rest
        for i in range(N):
            order = np.lexsort((np.arange(V), -logits[bb, i].astype(np.float64)))
            assert second[bb, i] == order[1]
    hb, wb = W.f32_to_bf16_bits(h), W.f32_to_bf16_bits(w)                # the same numbers as bf16
    assert np.array_equal(oracle.head_argmax(hb, wb)[0], amax)


def test_single_token_vocabulary_and_strided_hidden(oracle):
    rng = np.random.default_rng(8)
    h_big = rng.normal(size=(2, 4, 3, 16)).astype(np.float32)            # hidden states inside a wider buffer
    h = h_big[:, :, 1, :]
    w = rng.normal(size=(1, 16)).astype(np.float32)
    amax, _, gap, second = oracle.head_argmax(h, w)
    assert np.all(amax == 0) and np.all(np.isinf(gap)) and np.all(second == -1)
    w9 = rng.normal(size=(9, 16)).astype(np.float32)
    a1 = oracle.head_argmax(h, w9)[0]
    a2 = oracle.head_argmax(np.ascontiguousarray(h), w9)[0]
    assert np.array_equal(a1, a2)
