"""Pins of the oracle's tree attention against things other than itself.

SpecVLM Sec. 3.1 (one-pass verification) and Sec. 4.1 (tree attention) fix the
operation only by name, so the pins are: textbook causal attention (chain tree),
plain decode attention (one node), a numpy brute force with a materialised mask,
a hand-worked fixture, closed forms and mask-leak detectors.
"""
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_fixture(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(x) for x in vals]
    return out


def py_ancestor_mask(parent):
    """Ancestor-or-self matrix by walking parent links in pure Python."""
    n = len(parent)
    m = np.zeros((n, n), dtype=bool)
    for i in range(n):
        t = i
        while t != -1:
            m[i, t] = True
            t = int(parent[t])
    return m


def brute_force(q, k, v, P, parent, n, scale, hk_of_h):
    """Dense masked softmax with a materialised [n, P+n] mask (numpy/scipy, float64).
    q [n,H,D], k/v [Hkv,S,D] float64 -> o [n,H,D], lse [H,n]."""
    H, D = q.shape[1], q.shape[2]
    S = P + n
    mask = np.zeros((n, S), dtype=bool)
    mask[:, :P] = True
    mask[:, P:] = py_ancestor_mask(parent[:n])
    o = np.zeros((n, H, D))
    lse = np.zeros((H, n))
    for h in range(H):
        kk, vv = k[hk_of_h(h), :S], v[hk_of_h(h), :S]
        s = scale * (q[:, h, :] @ kk.T)
        s = np.where(mask, s, -np.inf)
        o[:, h, :] = softmax(s, axis=1) @ np.where(np.isfinite(vv), vv, 0.0)
        lse[h] = logsumexp(s, axis=1)
    return o, lse


def make_case(rng, dtype, B, Hq, Hkv, D, N, P_list, tree="random", depth=4, S_extra=5):
    q = W.normal(rng, (B, N, Hq, D), 1.0, dtype)
    S_cap = max(P_list) + N + S_extra
    k = W.normal(rng, (B, Hkv, S_cap, D), 1.0, dtype)
    v = W.normal(rng, (B, Hkv, S_cap, D), 1.0, dtype)
    if tree == "chain":
        parent = np.stack([W.chain_tree(N) for _ in range(B)])
    else:
        parent = np.stack([W.random_tree(rng, N, depth) for _ in range(B)])
    return q, k, v, np.array(P_list, dtype=np.int32), parent


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_tree_is_causal_attention(oracle, dtype):
    """A chain-shaped tree is ordinary causal attention of N new tokens over P+N keys."""
    rng = np.random.default_rng(1)
    B, H, D, N, P = 2, 3, 16, 7, 11
    q, k, v, Pl, parent = make_case(rng, dtype, B, H, H, D, N, [P, P - 4], tree="chain")
    o, lse = oracle.tree_attn(q, k, v, Pl, parent)
    qf, kf, vf = W.as_f64(q), W.as_f64(k), W.as_f64(v)
    for b in range(B):
        Pb = int(Pl[b])
        S = Pb + N
        for h in range(H):
            s = (qf[b, :, h, :] @ kf[b, h, :S].T) / math.sqrt(D)
            causal = np.arange(S)[None, :] <= (Pb + np.arange(N))[:, None]
            s = np.where(causal, s, -np.inf)
            ref = softmax(s, axis=1) @ vf[b, h, :S]
            np.testing.assert_allclose(o[b, :, h, :], ref, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(lse[b, h], logsumexp(s, axis=1), rtol=1e-12)


def test_single_node_is_decode_attention(oracle):
    """A one-node tree is plain decode attention over P+1 keys."""
    rng = np.random.default_rng(2)
    B, H, D, P = 3, 2, 32, 20
    q, k, v, Pl, parent = make_case(rng, "bf16", B, H, H, D, 1, [P, 1, 0])
    o, lse = oracle.tree_attn(q, k, v, Pl, parent)
    qf, kf, vf = W.as_f64(q), W.as_f64(k), W.as_f64(v)
    for b in range(B):
        S = int(Pl[b]) + 1
        for h in range(H):
            s = kf[b, h, :S] @ qf[b, 0, h] / math.sqrt(D)
            ref = softmax(s) @ vf[b, h, :S]
            np.testing.assert_allclose(o[b, 0, h], ref, rtol=1e-12, atol=1e-13)
            assert abs(lse[b, h, 0] - logsumexp(s)) < 1e-12


@pytest.mark.parametrize("seed", range(6))
def test_matches_materialised_mask_brute_force(oracle, seed):
    """Random small trees, GQA, ragged node counts, explicit scale, empty prefix."""
    rng = np.random.default_rng(100 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    B, Hq, Hkv, D, N = 3, 4, (2 if seed % 3 else 4), 8, 9
    P_list = [int(rng.integers(0, 12)) for _ in range(B)]
    P_list[seed % B] = 0
    q, k, v, Pl, parent = make_case(rng, dtype, B, Hq, Hkv, D, N, P_list)
    num_nodes = np.array([N, 1 + seed % N, max(1, N - 2)], dtype=np.int32)
    scale = 0.37
    # poison everything the definition must not read
    poison = W.NAN_BITS_BF16 if dtype == "bf16" else np.float32(np.nan)
    for b in range(B):
        k[b, :, P_list[b] + num_nodes[b]:, :] = poison
        v[b, :, P_list[b] + num_nodes[b]:, :] = poison
    o, lse = oracle.tree_attn(q, k, v, Pl, parent, num_nodes, scale=scale)
    qf, kf, vf = W.as_f64(q), W.as_f64(k), W.as_f64(v)
    g = Hq // Hkv
    for b in range(B):
        n = int(num_nodes[b])
        ref_o, ref_lse = brute_force(qf[b, :n], kf[b], vf[b], P_list[b], parent[b], n, scale,
                                     lambda h: h // g)
        np.testing.assert_allclose(o[b, :n], ref_o, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse[b, :, :n], ref_lse, rtol=1e-11, atol=1e-12)
        assert np.all(o[b, n:] == 0.0)


def test_paged_equals_contiguous(oracle):
    """Reading through a block table gives the same numbers as the contiguous cache."""
    rng = np.random.default_rng(7)
    B, H, D, N, bs = 2, 2, 8, 6, 16
    P_list = [21, 40]
    q, k, v, Pl, parent = make_case(rng, "bf16", B, H, H, D, N, P_list, S_extra=0)
    S_cap = W.round_up(k.shape[2], bs)
    kc = np.zeros((B, H, S_cap, D), dtype=np.uint16)
    vc = np.zeros_like(kc)
    kc[:, :, :k.shape[2]] = k
    vc[:, :, :v.shape[2]] = v
    table, nb = W.block_table(rng, B, S_cap // bs, spare=0.3)
    kp = np.full((nb, H, bs, D), W.NAN_BITS_BF16, dtype=np.uint16)
    vp = np.full_like(kp, W.NAN_BITS_BF16)
    for b in range(B):
        for blk in range(S_cap // bs):
            kp[table[b, blk]] = kc[b, :, blk * bs:(blk + 1) * bs]
            vp[table[b, blk]] = vc[b, :, blk * bs:(blk + 1) * bs]
    o1, l1 = oracle.tree_attn(q, kc, vc, Pl, parent)
    o2, l2 = oracle.tree_attn(q, kp, vp, Pl, parent, block_table=table, block_size=bs)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_hand_worked_uniform_fixture(oracle):
    fx = read_fixture("attn_uniform_weights.txt")
    P = int(fx["P"][0])
    parent = np.array(fx["parent"], dtype=np.int32)[None]
    N, D = parent.shape[1], 2
    vrows = np.array(fx["v"], dtype=np.float32).reshape(1, 1, P + N, D)
    k = np.random.default_rng(3).standard_normal((1, 1, P + N, D)).astype(np.float32)
    q = np.zeros((1, N, 1, D), dtype=np.float32)
    o, lse = oracle.tree_attn(q, k, vrows, [P], parent)
    np.testing.assert_allclose(o.reshape(N, D), np.array(fx["o"]).reshape(N, D), rtol=1e-14)
    np.testing.assert_allclose(lse.reshape(N), np.log(np.array(fx["visible"])), rtol=1e-14)
    # the same through bf16 storage (all fixture values are exactly representable)
    o16, _ = oracle.tree_attn(W.f32_to_bf16_bits(q), W.f32_to_bf16_bits(k),
                              W.f32_to_bf16_bits(vrows), [P], parent)
    np.testing.assert_allclose(o16.reshape(N, D), np.array(fx["o"]).reshape(N, D), rtol=1e-14)


def test_two_key_closed_form_and_scale(oracle):
    """Scores a_j on the first coordinate: weights are exp(scale*2*a_j) / sum; default
    scale is 1/sqrt(D)."""
    D, P = 4, 1
    parent = np.array([[-1, 0]], dtype=np.int32)
    q = np.zeros((1, 2, 1, D), dtype=np.float32)
    q[0, :, 0, 0] = 2.0
    k = np.zeros((1, 1, 3, D), dtype=np.float32)
    k[0, 0, :, 0] = [0.0, 1.0, -3.0]
    k[0, 0, :, 1] = [5.0, -7.0, 9.0]          # orthogonal to q: must not matter
    v = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 0, 1.0, 0]], dtype=np.float32).reshape(1, 1, 3, D)
    o, lse = oracle.tree_attn(q, k, v, [P], parent)
    e0, e1, e2 = 1.0, math.e, math.exp(-3.0)          # scale 0.5 * q 2 * a
    np.testing.assert_allclose(o[0, 0, 0], [e0 / (e0 + e1), e1 / (e0 + e1), 0, 0], rtol=1e-14)
    z = e0 + e1 + e2
    np.testing.assert_allclose(o[0, 1, 0], [e0 / z, e1 / z, e2 / z, 0], rtol=1e-14)
    np.testing.assert_allclose(lse[0, 0], [math.log(e0 + e1), math.log(z)], rtol=1e-14)
    o2, _ = oracle.tree_attn(q, k, v, [P], parent, scale=1.0)
    z2 = 1 + math.exp(2.0)
    np.testing.assert_allclose(o2[0, 0, 0], [1 / z2, math.exp(2.0) / z2, 0, 0], rtol=1e-14)


@pytest.mark.parametrize("seed", range(3))
def test_path_extraction_reduces_tree_to_chain(oracle, seed):
    """Node i's output equals the last row of a chain run on its root path."""
    rng = np.random.default_rng(40 + seed)
    H, D, N, P = 2, 16, 12, 9
    q, k, v, Pl, parent = make_case(rng, "bf16", 1, H, H, D, N, [P], depth=5, S_extra=0)
    o, lse = oracle.tree_attn(q, k, v, Pl, parent)
    for i in range(N):
        path = []
        t = i
        while t != -1:
            path.append(t)
            t = int(parent[0, t])
        path = path[::-1]
        n = len(path)
        q2 = q[:, path]
        k2 = np.concatenate([k[:, :, :P], k[:, :, [P + j for j in path]]], axis=2)
        v2 = np.concatenate([v[:, :, :P], v[:, :, [P + j for j in path]]], axis=2)
        o2, lse2 = oracle.tree_attn(np.ascontiguousarray(q2), np.ascontiguousarray(k2),
                                    np.ascontiguousarray(v2), Pl, W.chain_tree(n)[None])
        np.testing.assert_allclose(o[0, i], o2[0, n - 1], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[0, :, i], lse2[0, :, n - 1], rtol=1e-12)


def test_relabelling_permutes_outputs(oracle):
    """Another topological numbering of the same tree permutes the rows of o."""
    rng = np.random.default_rng(9)
    H, D, N, P = 2, 8, 10, 6
    q, k, v, Pl, parent = make_case(rng, "f32", 1, H, H, D, N, [P], depth=4, S_extra=0)
    o, _ = oracle.tree_attn(q, k, v, Pl, parent)
    depth = W.tree_depths(parent[0])
    order = sorted(range(N), key=lambda i: (depth[i], -i))      # new -> old, still topological
    new_of_old = {old: new for new, old in enumerate(order)}
    parent2 = np.array([[-1 if parent[0, old] < 0 else new_of_old[int(parent[0, old])]
                         for old in order]], dtype=np.int32)
    q2 = np.ascontiguousarray(q[:, order])
    k2, v2 = k.copy(), v.copy()
    k2[:, :, P:P + N] = k[:, :, [P + old for old in order]]
    v2[:, :, P:P + N] = v[:, :, [P + old for old in order]]
    o2, _ = oracle.tree_attn(q2, k2, v2, Pl, parent2)
    np.testing.assert_allclose(o2[0], o[0, order], rtol=1e-12, atol=1e-14)


def test_constant_v_and_mask_leaks(oracle):
    """V == 1 gives o == 1 exactly; huge V in invisible tree slots changes nothing."""
    rng = np.random.default_rng(11)
    H, D, N, P = 2, 8, 9, 5
    q, k, v, Pl, parent = make_case(rng, "f32", 1, H, H, D, N, [P], depth=3, S_extra=3)
    ones = np.ones_like(v)
    o, _ = oracle.tree_attn(q, k, ones, Pl, parent)
    np.testing.assert_allclose(o, 1.0, rtol=0, atol=4e-16)
    base, _ = oracle.tree_attn(q, k, v, Pl, parent)
    anc = py_ancestor_mask(parent[0])
    for i in range(N):
        v2 = v.copy()
        k2 = k.copy()
        for j in range(N):
            if not anc[i, j]:
                v2[0, :, P + j] = 1e4
                k2[0, :, P + j] = 50.0
        v2[0, :, P + N:] = np.nan
        o2, _ = oracle.tree_attn(q, k2, v2, Pl, parent)
        assert np.array_equal(o2[0, i], base[0, i])


def test_ancestors_and_malformed_trees(oracle):
    parent = np.array([-1, 0, 0, 1, 3, 2], dtype=np.int32)
    anc, depth = oracle.ancestors(parent)
    assert np.array_equal(anc.astype(bool), py_ancestor_mask(parent))
    assert depth.tolist() == [0, 1, 1, 2, 3, 2]
    for bad in ([0, 0, 1], [-1, 1, 0], [-1, 0, 5], [-1, -1]):
        with pytest.raises(ValueError):
            oracle.ancestors(np.array(bad, dtype=np.int32))
