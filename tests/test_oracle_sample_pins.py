"""Pins of the oracle's argmax, acceptance walk and KV compaction.

SpecVLM Sec. 3.1: the target verifies the drafted tokens in one pass and the
incorrect ones are discarded, losslessly (abstract; Sec. 4.1 "Metrics"); the
evaluation is greedy at temperature 0.  sigma's closed form is from Sec. 3.1.
"""
import os

import numpy as np
import pytest

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
            out[key] = [int(x) for x in vals]
    return out


# ----------------------------------------------------------------- argmax
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_argmax_matches_numpy_first_occurrence(oracle, dtype):
    rng = np.random.default_rng(5)
    B, N, V = 2, 7, 3001
    logits = W.normal(rng, (B, N, V), 2.0, dtype)
    vals = W.as_f64(logits)
    got = oracle.node_argmax(logits)
    assert np.array_equal(got, np.argmax(vals, axis=2))          # numpy: first maximal index
    if dtype == "bf16":                                           # ties must really occur
        ties = (vals == vals.max(axis=2, keepdims=True)).sum(axis=2)
        assert ties.max() >= 1


def test_argmax_ties_zero_signs_inf_and_ragged(oracle):
    V = 50
    x = np.full((1, 6, V), -1.0, dtype=np.float32)
    x[0, 0, [7, 30, 49]] = 3.0                       # three-way tie -> 7
    x[0, 1, :] = -np.inf                             # all -inf -> 0
    x[0, 2, :] = -np.inf
    x[0, 2, 41] = -1e30                              # single finite value
    x[0, 3, :] = -0.0
    x[0, 3, 5] = 0.0                                 # -0 == +0 -> index 0
    x[0, 4, 49] = np.inf                             # +inf at the last index
    x[0, 4, 20] = 3e38
    x[0, 5, 0] = 9.0                                 # row beyond num_nodes
    got = oracle.node_argmax(x, num_nodes=[5])
    assert got[0].tolist() == [7, 0, 41, 0, 49, -1]
    got16 = oracle.node_argmax(W.f32_to_bf16_bits(x), num_nodes=[5])
    assert got16[0].tolist() == [7, 0, 41, 0, 49, -1]


def test_argmax_strided_rows(oracle):
    rng = np.random.default_rng(6)
    big = rng.standard_normal((2, 5, 300)).astype(np.float32)
    view = big[:, :, :257]                           # row stride 300, V = 257
    assert np.array_equal(oracle.node_argmax(view), np.argmax(view, axis=2))


# ----------------------------------------------------------------- accept
def enumerate_best_path(parent, tok, amax, n):
    """Exhaustive: test every node's whole root path, keep the deepest, lowest index on ties."""
    best, best_path = 0, [0]
    for i in range(n):
        path = [i]
        while parent[path[-1]] != -1:
            path.append(int(parent[path[-1]]))
        path = path[::-1]
        good = all(tok[path[j + 1]] == amax[path[j]] for j in range(len(path) - 1))
        if good and len(path) > len(best_path):
            best, best_path = i, path
    return best_path


def test_accept_hand_worked_fixture(oracle):
    fx = read_fixture("accept_worked.txt")
    parent = np.array([fx["parent"]], dtype=np.int32)
    m, path, bonus, committed = oracle.tree_accept(parent, [fx["draft_tok"]], [fx["amax"]], path_cap=5)
    assert m[0] == fx["accept_len"][0]
    assert path[0].tolist() == fx["path"] + [-1] * (5 - len(fx["path"]))
    assert bonus[0] == fx["bonus"][0]
    assert committed[0].tolist() == fx["committed"] + [-1] * (5 - len(fx["committed"]))


@pytest.mark.parametrize("seed", range(8))
def test_accept_matches_exhaustive_enumeration(oracle, seed):
    """Tiny vocab so that equal sibling tokens and multi-level matches are frequent."""
    rng = np.random.default_rng(200 + seed)
    B, N, V = 64, 10, 3
    parent = np.stack([W.random_tree(rng, N, 4) for _ in range(B)])
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    amax = rng.integers(0, V, size=(B, N)).astype(np.int32)
    num_nodes = rng.integers(1, N + 1, size=B).astype(np.int32)
    m, path, bonus, committed = oracle.tree_accept(parent, tok, amax, num_nodes, path_cap=6)
    depths_seen = set()
    for b in range(B):
        ref = enumerate_best_path(parent[b], tok[b], amax[b], int(num_nodes[b]))
        assert m[b] == len(ref) - 1
        assert path[b, :len(ref)].tolist() == ref and np.all(path[b, len(ref):] == -1)
        assert bonus[b] == amax[b, ref[-1]]
        assert committed[b, :len(ref)].tolist() == [int(tok[b, t]) for t in ref[1:]] + [int(amax[b, ref[-1]])]
        depths_seen.add(len(ref) - 1)
    assert len(depths_seen) >= 3


@pytest.mark.parametrize("name", ["C1", "C2", "C5"])
def test_accept_is_lossless_on_workload_trees(oracle, name):
    """Committed tokens equal what token-by-token greedy decoding emits from the same
    logits; no child of the last accepted node carries the bonus token."""
    cfg = W.CONFIGS[name]
    tb = W.make_trees(cfg)
    amax = oracle.node_argmax(tb.logits)
    m, path, bonus, committed = oracle.tree_accept(tb.parent, tb.draft_tok, amax, path_cap=cfg.depth + 1)
    for b in range(cfg.B):
        par, tok = tb.parent[b], tb.draft_tok[b]
        p = [int(t) for t in path[b] if t >= 0]
        assert len(p) == m[b] + 1 and p[0] == 0
        for j in range(len(p) - 1):
            assert par[p[j + 1]] == p[j] and tok[p[j + 1]] == amax[b, p[j]]
        kids = [i for i in range(cfg.N) if par[i] == p[-1]]
        assert all(tok[c] != amax[b, p[-1]] for c in kids)
        if cfg.tree == "eagle":                       # sibling tokens distinct: greedy walk is unique
            cur, emitted = 0, []
            while True:
                t = int(amax[b, cur])
                emitted.append(t)
                nxt = [i for i in range(cfg.N) if par[i] == cur and tok[i] == t]
                if not nxt:
                    break
                cur = nxt[0]
            assert committed[b, :m[b] + 1].tolist() == emitted
    if name != "C1":
        assert m.max() >= 1


def test_sigma_closed_form_fixture_values():
    with open(os.path.join(GOLD, "sigma_closed_form.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for a, g, s in rows:
        a, g, s = float(a), int(g), float(s)
        assert abs(a * (1 - a ** g) / (1 - a) - s) < 1e-12


@pytest.mark.parametrize("alpha,gamma", [(0.5, 3), (0.75, 6), (0.3, 5)])
def test_chain_acceptance_follows_sigma_closed_form(oracle, alpha, gamma):
    """Chains with i.i.d. per-token match probability alpha: mean accepted drafts ->
    alpha (1 - alpha^gamma) / (1 - alpha)."""
    rng = np.random.default_rng(77)
    B, N, V = 40000, gamma + 1, 1000
    parent = np.tile(W.chain_tree(N), (B, 1))
    amax = rng.integers(0, V, size=(B, N)).astype(np.int32)
    tok = np.zeros((B, N), dtype=np.int32)
    hit = rng.random((B, N)) < alpha
    tok[:, 1:] = np.where(hit[:, 1:], amax[:, :-1], (amax[:, :-1] + 1 + rng.integers(0, V - 1, size=(B, N - 1))) % V)
    m, _, _, _ = oracle.tree_accept(parent, tok, amax, path_cap=N)
    sigma = alpha * (1 - alpha ** gamma) / (1 - alpha)
    assert abs(m.mean() - sigma) < 4 * m.std() / np.sqrt(B)


def test_accept_relabelling_keeps_committed_tokens(oracle):
    cfg = W.CONFIGS["C2"]
    tb = W.make_trees(cfg)
    amax = oracle.node_argmax(tb.logits)
    _, _, _, committed = oracle.tree_accept(tb.parent, tb.draft_tok, amax, path_cap=8)
    par = tb.parent[0]
    depth = W.tree_depths(par)
    order = sorted(range(cfg.N), key=lambda i: (depth[i], -i))
    new_of_old = {old: new for new, old in enumerate(order)}
    par2 = np.array([[-1 if par[o] < 0 else new_of_old[int(par[o])] for o in order]], dtype=np.int32)
    _, _, _, committed2 = oracle.tree_accept(par2, tb.draft_tok[:, order], amax[:, order], path_cap=8)
    assert np.array_equal(committed, committed2)


def test_accept_rejects_bad_input(oracle):
    with pytest.raises(ValueError):
        oracle.tree_accept([[-1, 1, 0]], [[0, 0, 0]], [[0, 0, 0]])
    with pytest.raises(ValueError):                      # path longer than path_cap
        oracle.tree_accept([[-1, 0, 1]], [[0, 5, 5]], [[5, 5, 5]], path_cap=2)


# ----------------------------------------------------------------- compaction
def test_compact_hand_worked_fixture(oracle):
    fx = read_fixture("accept_worked.txt")
    P = fx["P"][0]
    L, H, D, S = 2, 2, 4, P + 8
    rng = np.random.default_rng(1)
    k = rng.integers(0, 65536, size=(L, 1, H, S, D), dtype=np.uint16)
    v = rng.integers(0, 65536, size=(L, 1, H, S, D), dtype=np.uint16)
    k0, v0 = k.copy(), v.copy()
    path = np.array([fx["path"] + [-1, -1]], dtype=np.int32)
    newp, moved = oracle.kv_compact(k, v, [P], path, [fx["accept_len"][0]])
    assert newp[0] == fx["new_prefix"][0]
    assert moved[0, :3].reshape(-1).tolist() == fx["moved"] and np.all(moved[0, 3:] == -1)
    for src, dst in zip(fx["moved"][0::2], fx["moved"][1::2]):
        assert np.array_equal(k[:, 0, :, dst], k0[:, 0, :, src])
        assert np.array_equal(v[:, 0, :, dst], v0[:, 0, :, src])
    assert np.array_equal(k[:, :, :, :P], k0[:, :, :, :P])


@pytest.mark.parametrize("paged", [False, True])
def test_compact_gather_semantics_with_overlapping_moves(oracle, paged):
    """Path [0,2,3]: slot P+2 is both a destination (of a_2=3) and a source (for j=1);
    the result must be a gather from the OLD cache.  Checked against numpy fancy indexing."""
    rng = np.random.default_rng(3)
    L, B, H, D, bs = 3, 3, 2, 8, 16
    P = np.array([5, 30, 16], dtype=np.int32)
    paths = np.array([[0, 2, 3, -1, -1], [0, 1, 2, 3, 4], [0, -1, -1, -1, -1]], dtype=np.int32)
    m = np.array([2, 4, 0], dtype=np.int32)
    S_cap = 48
    if paged:
        table, nb = W.block_table(rng, B, S_cap // bs, spare=0.5)
        k = rng.integers(0, 65536, size=(L, nb, H, bs, D), dtype=np.uint16)
        v = rng.integers(0, 65536, size=(L, nb, H, bs, D), dtype=np.uint16)
        def row(arr, b, slot):
            return arr[:, table[b, slot // bs], :, slot % bs]
    else:
        table = None
        k = rng.integers(0, 65536, size=(L, B, H, S_cap, D), dtype=np.uint16)
        v = rng.integers(0, 65536, size=(L, B, H, S_cap, D), dtype=np.uint16)
        def row(arr, b, slot):
            return arr[:, b, :, slot]
    k0, v0 = k.copy(), v.copy()
    newp, moved = oracle.kv_compact(k, v, P, paths, m, block_table=table, block_size=bs)
    assert newp.tolist() == (P + m + 1).tolist()
    touched = np.zeros(k.shape, dtype=bool)
    for b in range(B):
        for j in range(m[b] + 1):
            assert moved[b, j].tolist() == [P[b] + paths[b, j], P[b] + j]
            assert np.array_equal(row(k, b, P[b] + j), row(k0, b, P[b] + paths[b, j]))
            assert np.array_equal(row(v, b, P[b] + j), row(v0, b, P[b] + paths[b, j]))
            row(touched, b, P[b] + j)[...] = True
    assert np.array_equal(k[~touched], k0[~touched]) and np.array_equal(v[~touched], v0[~touched])


def test_compact_fp32_rows_and_aliasing_of_prefix(oracle):
    rng = np.random.default_rng(4)
    k = rng.standard_normal((1, 1, 1, 12, 4)).astype(np.float32)
    v = rng.standard_normal((1, 1, 1, 12, 4)).astype(np.float32)
    k0 = k.copy()
    newp, _ = oracle.kv_compact(k, v, [4], [[0, 3, 5]], [2])
    assert newp[0] == 7
    assert np.array_equal(k[0, 0, 0, 4:7], k0[0, 0, 0, [4, 7, 9]])
