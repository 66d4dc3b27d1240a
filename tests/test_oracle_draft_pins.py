"""Pins of the oracle's draft-side tree growth (SpecVLM Sec. 4.1: the draft grows an EAGLE-2 style
token tree -- Top-K 10, 60 tokens in total, depth 7 -- which the target then verifies).

The paper gives the three numbers only; the oracle states the growth rule (value of a node = sum
of the draft's log-probabilities on its root path, Top-K expansion of the most valuable nodes of
a level, the most valuable candidates overall form the tree).  Pinned here by a hand-worked
fixture, closed forms, numpy/scipy library routines and, for the whole growth, by brute force:
with every candidate expanded the tree must consist of the most probable token sequences.
"""
import itertools
import os

import numpy as np
import pytest
from scipy.special import log_softmax, logsumexp

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


def ln32(p):
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def test_hand_worked_growth(oracle):
    fx = read_fixture("draft_growth_worked.txt")
    lv = [ln32(fx["root_probs"]).reshape(1, 1, 4),
          np.stack([ln32(fx["row0_probs"]), ln32(fx["row1_probs"])]).reshape(1, 2, 4)]
    r = oracle.grow_tree(lv, [int(fx["root_token"][0])], K=2, width=2, N_max=5)
    assert r["cand_token"][0].tolist() == [int(x) for x in fx["cand_token"]]
    assert r["cand_parent"][0].tolist() == [int(x) for x in fx["cand_parent"]]
    np.testing.assert_allclose(np.exp(r["cand_score"][0].astype(np.float64)), fx["cand_value"], rtol=1e-6)
    assert r["parent"][0].tolist() == [int(x) for x in fx["parent"]]
    assert r["draft_tok"][0].tolist() == [int(x) for x in fx["draft_tok"]]
    assert r["node_cand"][0].tolist() == [int(x) for x in fx["node_cand"]]
    assert r["num_nodes"][0] == int(fx["num_nodes"][0])
    assert abs(r["final_gap"][0] - np.log(fx["gap_ln"][0])) < 1e-6


def test_hand_worked_selection_with_ties(oracle):
    fx = read_fixture("draft_growth_worked.txt")
    sel, cnt, gap = oracle.tree_select(np.array([fx["select_score"]], dtype=np.float32), int(fx["select_M"][0]))
    assert sel[0].tolist() == [int(x) for x in fx["select_sel"]]
    assert cnt[0] == 3 and gap[0] == fx["select_gap"][0]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_topk_against_library_routines(oracle, dtype):
    """Top-K tokens = stable argsort of the negated logits (equal logits keep the lower token
    first); scores = cum + scipy's log_softmax; lse = scipy's logsumexp."""
    rng = np.random.default_rng(42)
    R, V, K = 7, 300, 10
    lg = W.normal(rng, (R, V), 2.0, dtype)
    x = W.as_f64(lg)
    cum = -rng.random(R) * 5
    score, token, lse = oracle.topk_logprob(lg, K, cum)
    want_tok = np.argsort(-x, axis=1, kind="stable")[:, :K]
    assert np.array_equal(token, want_tok)          # bf16 rows hold many equal logits
    want = cum[:, None] + np.take_along_axis(log_softmax(x, axis=1), want_tok, axis=1)
    np.testing.assert_allclose(score, want, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, logsumexp(x, axis=1), rtol=0, atol=1e-12)
    s0, t0, _ = oracle.topk_logprob(lg, K)           # cum omitted = 0
    np.testing.assert_allclose(s0, want - cum[:, None], rtol=0, atol=1e-12)
    assert np.array_equal(t0, want_tok)


def test_topk_closed_forms(oracle):
    V, K = 64, 5
    flat = np.full((1, V), 3.25, dtype=np.float32)                       # uniform: every score is -ln V
    score, token, lse = oracle.topk_logprob(flat, K)
    assert token[0].tolist() == list(range(K))
    np.testing.assert_allclose(score[0], -np.log(V), atol=1e-14)
    np.testing.assert_allclose(lse[0], 3.25 + np.log(V), atol=1e-14)
    rng = np.random.default_rng(3)                                       # K = V: probabilities sum to one
    lg = rng.normal(0, 3, size=(4, 40)).astype(np.float32)
    score, token, _ = oracle.topk_logprob(lg, 40)
    np.testing.assert_allclose(np.exp(score).sum(axis=1), 1.0, atol=1e-13)
    assert np.all(np.diff(score, axis=1) <= 0)                           # greater first
    assert all(sorted(t.tolist()) == list(range(40)) for t in token)
    two = np.array([[0.0, np.log(3.0)]], dtype=np.float64).astype(np.float32)   # p = 1/4, 3/4
    score, token, _ = oracle.topk_logprob(two, 2, np.array([-1.0]))
    assert token[0].tolist() == [1, 0]
    np.testing.assert_allclose(np.exp(score[0] + 1.0), [0.75, 0.25], rtol=1e-7)
    huge = np.array([[1e4, 1e4 - 1.0, -1e4]], dtype=np.float32)           # no overflow
    score, _, lse = oracle.topk_logprob(huge, 3)
    np.testing.assert_allclose(lse[0], 1e4 + np.log1p(np.exp(-1.0)), rtol=1e-15)
    assert np.isfinite(score).all()
    with pytest.raises(ValueError):
        oracle.topk_logprob(two, 3)                                       # K > V


def test_top1_is_the_greedy_token(oracle):
    rng = np.random.default_rng(9)
    lg = W.normal(rng, (1, 12, 500), 2.0, "bf16")
    _, token, _ = oracle.topk_logprob(lg.reshape(12, 500), 1)
    assert np.array_equal(token[:, 0], oracle.node_argmax(lg)[0])


@pytest.mark.parametrize("seed", range(4))
def test_select_against_lexsort(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    B, C, M = 6, 100, 10
    score = np.round(rng.normal(0, 1, size=(B, C)) * 4).astype(np.float32) / 4      # many exact ties
    num = rng.integers(1, C + 1, size=B).astype(np.int32)
    num[0], num[1] = C, 3                                                            # full and shorter than M
    sel, cnt, gap = oracle.tree_select(score, M, num)
    for b in range(B):
        c = int(num[b])
        order = np.lexsort((np.arange(c), -score[b, :c].astype(np.float64)))         # score down, index up
        win = np.sort(order[:M])
        assert cnt[b] == min(M, c)
        assert sel[b, :cnt[b]].tolist() == win.tolist() and np.all(sel[b, cnt[b]:] == -1)
        if c > M:
            assert gap[b] == float(score[b, order[M - 1]]) - float(score[b, order[M]])
        else:
            assert gap[b] == np.inf


def _paths_of(parent, tok, n):
    out = set()
    for i in range(1, n):
        seq, t = [], i
        while t > 0:
            seq.append(int(tok[t]))
            t = int(parent[t])
        out.add(tuple(reversed(seq)))
    return out


@pytest.mark.parametrize("seed", range(5))
def test_exhaustive_growth_keeps_the_most_probable_sequences(oracle, seed):
    """With every candidate expanded (width >= candidates per level, K = V) the growth scores all
    token sequences up to the depth, so the tree must be exactly the N_max - 1 sequences of
    greatest joint draft probability -- computed here by enumeration, independently."""
    rng = np.random.default_rng(700 + seed)
    V, depth, N_max = 3, 3, 14
    rows = [1, 3, 9]
    lv = [rng.normal(0, 1.2, size=(1, r, V)).astype(np.float32) for r in rows]
    r = oracle.grow_tree(lv, [5], K=V, width=9, N_max=N_max)
    # which logits row conditions on which token sequence: rows follow the candidate order of the
    # previous level, i.e. parents in order, each parent's tokens by decreasing probability
    lp = [log_softmax(l[0].astype(np.float64), axis=1) for l in lv]
    order = lambda row: np.argsort(-row, kind="stable")
    seqs = {}
    level = [((), 0.0)]
    for d in range(depth):
        nxt = []
        for row, (seq, s) in enumerate(level):
            for t in order(lp[d][row]):
                nxt.append((seq + (int(t),), s + lp[d][row][t]))
        for seq, s in nxt:
            seqs[seq] = s
        level = nxt
    ranked = sorted(seqs.items(), key=lambda kv: -kv[1])
    assert ranked[N_max - 2][1] - ranked[N_max - 1][1] > 1e-5              # the cut is not a near-tie
    want = {seq for seq, _ in ranked[:N_max - 1]}
    got = _paths_of(r["parent"][0], r["draft_tok"][0], int(r["num_nodes"][0]))
    assert got == want
    assert r["num_nodes"][0] == N_max and r["draft_tok"][0, 0] == 5
    # node values are the joint log-probabilities of their sequences
    for j in range(1, N_max):
        seq, t = [], j
        while t > 0:
            seq.append(int(r["draft_tok"][0, t])); t = int(r["parent"][0, t])
        assert abs(float(r["cand_score"][0, r["node_cand"][0, j]]) - seqs[tuple(reversed(seq))]) < 1e-5


@pytest.mark.parametrize("seed", range(3))
def test_growth_invariants_at_paper_size(oracle, seed):
    """Top-K 10, ten nodes expanded per level, depth 7, 60 tokens (Sec. 4.1)."""
    rng = np.random.default_rng(900 + seed)
    B, V, K, depth, N = 3, 2000, 10, 7, 60
    lv = [W.normal(rng, (B, 1 if d == 0 else K, V), 2.0, "bf16") for d in range(depth)]
    r = oracle.grow_tree(lv, [1, 2, 3], K=K, width=K, N_max=N)
    C = K + (depth - 1) * K * K
    assert r["cand_score"].shape == (B, C)
    for b in range(B):
        par, tok, nc = r["parent"][b], r["draft_tok"][b], r["node_cand"][b]
        assert r["num_nodes"][b] == N and par[0] == -1 and np.all((par[1:] >= 0) & (par[1:] < np.arange(1, N)))
        sc = r["cand_score"][b]
        # a child never outscores its parent; selection is closed under "parent of"
        cp = r["cand_parent"][b]
        assert np.all(sc[cp >= 0] <= sc[cp[cp >= 0]])
        chosen = set(nc[1:].tolist())
        assert all(cp[c] < 0 or cp[c] in chosen for c in chosen)
        # the chosen are the N-1 best by (score, lower index): nobody left out beats the worst chosen
        rest = np.setdiff1d(np.arange(C), nc[1:])
        assert sc[rest].max() <= sc[nc[1:]].min()
        assert abs((sc[nc[1:]].min() - sc[rest].max()) - r["final_gap"][b]) < 1e-12
        # sibling tokens are distinct (Top-K of one distribution) and the tree reaches depth >= 2
        for node in range(N):
            kids = tok[1:][par[1:] == node]
            assert len(set(kids.tolist())) == len(kids)
        assert W.tree_depths(par).max() <= depth
        # tokens of the nodes are the candidates' tokens; parents map through node_cand
        assert np.array_equal(tok[1:], r["cand_token"][b][nc[1:]])
        for j in range(1, N):
            assert (cp[nc[j]] < 0 and par[j] == 0) or nc[par[j]] == cp[nc[j]]
        # each level's expanded nodes are the best `width` of the previous level's candidates
    for d, sel in enumerate(r["level_sel"]):
        base = 0 if d == 0 else K + (d - 1) * K * K
        cnt = K if d == 0 else K * K
        for b in range(B):
            rng_sc = r["cand_score"][b, base:base + cnt]
            assert np.all(np.diff(sel[b]) > 0) and sel[b].min() >= base and sel[b].max() < base + cnt
            left = np.setdiff1d(np.arange(cnt), sel[b] - base)
            if len(left):
                assert rng_sc[left].max() <= rng_sc[sel[b] - base].min()


def test_finalize_rejects_bad_candidates(oracle):
    score = np.array([[-1.0, -2.0, -0.5]], dtype=np.float32)
    tok = np.array([[4, 5, 6]], dtype=np.int32)
    with pytest.raises(ValueError):                       # a parent that does not precede its child
        oracle.tree_finalize(score, np.array([[-1, 2, 0]]), tok, [0], 4)
    with pytest.raises(ValueError):                       # child (c2, -0.5) chosen without its parent (c1, -2.0)
        oracle.tree_finalize(score, np.array([[-1, -1, 1]]), tok, [0], 3)
    par, t, nc, n, gap = oracle.tree_finalize(score, np.array([[-1, 0, 0]]), tok, [7], 8)   # fewer than N_max - 1
    assert n[0] == 4 and par[0].tolist() == [-1, 0, 1, 1, -1, -1, -1, -1] and t[0, :4].tolist() == [7, 4, 5, 6]
    assert gap[0] == np.inf
    par, t, nc, n, _ = oracle.tree_finalize(score, np.array([[-1, 0, 0]]), tok, [7], 1)     # root only
    assert n[0] == 1 and par[0].tolist() == [-1] and t[0].tolist() == [7]
