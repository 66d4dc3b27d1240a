"""Pins of the oracle's sampling-based acceptance walk (temperature > 0).

SpecVLM Sec. 3.1 names speculative sampling as the rule that discards drafted tokens and
gives sigma's closed form alpha(1-alpha^gamma)/(1-alpha); Sec. 4.1 evaluates temperature 1
and states that decoding stays lossless (the output follows the target's distribution).
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
            out[key] = [float(x) for x in vals]
    return out


def log_probs(p):
    with np.errstate(divide="ignore"):
        return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


@pytest.mark.parametrize("case", ["A", "B", "C"])
def test_hand_worked_fixture(oracle, case):
    fx = read_fixture("accept_sample_worked.txt")
    parent = np.array([fx["parent"]], dtype=np.int32)
    tok = np.array([fx["draft_tok"]], dtype=np.int32)
    logits = log_probs(fx["probs"]).reshape(1, 6, 3)
    m, path, bonus, committed, info = oracle.tree_accept_sample(
        parent, tok, logits, [fx[case + "_u_accept"]], fx[case + "_u_bonus"], path_cap=4)
    want_path = [int(x) for x in fx[case + "_path"]]
    want_comm = [int(x) for x in fx[case + "_committed"]]
    assert m[0] == int(fx[case + "_accept_len"][0])
    assert path[0].tolist() == want_path + [-1] * (4 - len(want_path))
    assert committed[0].tolist() == want_comm + [-1] * (4 - len(want_comm))
    assert bonus[0] == want_comm[-1]
    # the diagnostics that decide which requests a lower-precision evaluation is held to, hand-worked too
    # (inputs pass through float32: ln p, u)
    assert abs(info["margin_accept"][0] - fx[case + "_margin_accept"][0]) < 1e-6
    assert abs(info["margin_bonus"][0] - fx[case + "_margin_bonus"][0]) < 1e-6
    assert info["bonus_alt"][0] == int(fx[case + "_bonus_alt"][0])


def test_margins_against_cumulative_sums(oracle):
    """margin_accept, margin_bonus and bonus_alt by brute force: a root with a few leaf children over a
    small vocabulary (some tokens of probability 0, some children repeating a token), thresholds and CDF
    edges from numpy's cumulative sums in float64."""
    rng = np.random.default_rng(2509)
    for trial in range(400):
        V = int(rng.integers(2, 9))
        K = int(rng.integers(0, 5))                                   # children of the root, all leaves
        N = K + 1
        parent = np.array([[-1] + [0] * K], dtype=np.int32)
        logits = rng.normal(0.0, 1.5, size=(1, N, V)).astype(np.float32)
        dead = rng.random(V) < 0.25
        if dead.all():
            dead[int(rng.integers(0, V))] = False
        logits[0, :, dead] = -np.inf
        tok = np.concatenate([[0], rng.integers(-1, V + 1, size=K)]).astype(np.int32)[None]   # some out of range
        ua = rng.random((1, N), dtype=np.float32)
        ub = rng.random(1, dtype=np.float32)
        T = float(rng.choice([1.0, 0.5, 2.0]))
        m, path, bonus, committed, info = oracle.tree_accept_sample(parent, tok, logits, ua, ub, temperature=T, path_cap=4)

        def probs(row):
            z = np.exp((row.astype(np.float64) - row[np.isfinite(row)].max()) / T)
            return z / z.sum()

        p = probs(logits[0, 0])
        rejected = np.zeros(V, dtype=bool)
        margin, cur = 1.0, 0
        for c in range(1, N):
            x = int(tok[0, c])
            if not (0 <= x < V) or rejected[x]:
                continue                                             # rejected whatever the precision: not a comparison
            a = p[x] / (1.0 - p[rejected].sum())
            margin = min(margin, abs(float(ua[0, c]) - a))
            if float(ua[0, c]) < a:
                cur = c
                break
            rejected[x] = True
        if cur:                                                      # a leaf: its own distribution, nothing rejected
            p, rejected = probs(logits[0, cur]), np.zeros(V, dtype=bool)
        assert m[0] == (1 if cur else 0) and path[0, :2].tolist() == ([0, cur] if cur else [0, -1])
        assert abs(info["margin_accept"][0] - margin) < 1e-9
        live = np.nonzero(~rejected & (p > 0))[0]
        mass = p[live]
        edges = np.concatenate([[0.0], np.cumsum(mass)])             # token live[i] covers [edges[i], edges[i+1])
        t = float(ub[0]) * edges[-1]
        i = min(int(np.searchsorted(edges, t, side="right")) - 1, len(live) - 1)
        assert bonus[0] == live[i]
        d_lo, d_hi = (t - edges[i]) / edges[-1], (edges[i + 1] - t) / edges[-1]
        j = i - 1 if d_lo <= d_hi else i + 1
        if 0 <= j < len(live):
            assert info["bonus_alt"][0] == live[j]
            assert abs(info["margin_bonus"][0] - min(d_lo, d_hi)) < 1e-9
        else:                                                        # no token across the nearer edge
            assert info["bonus_alt"][0] == live[i] and info["margin_bonus"][0] == 1.0


def _tiny_tree():
    #        0
    #      / | \
    #     1  2  3       tokens 4, 1, 2
    #    / \    |
    #   4   5   6       tokens 0, 3 (under 1), 5 (under 3)
    parent = np.array([-1, 0, 0, 0, 1, 1, 3], dtype=np.int32)
    tok = np.array([0, 4, 1, 2, 0, 3, 5], dtype=np.int32)
    return parent, tok


@pytest.mark.parametrize("temperature", [1.0, 0.6])
def test_output_distribution_equals_the_targets(oracle, temperature):
    """Lossless: the first emitted token follows softmax(logits[root]/T), and after an accepted
    child the next emitted token follows that child's own distribution."""
    rng = np.random.default_rng(11815)
    parent, tok = _tiny_tree()
    V, N, B = 6, 7, 400_000
    base = rng.normal(0.0, 1.5, size=(N, V)).astype(np.float32)
    logits = np.broadcast_to(base, (B, N, V))
    ua = rng.random((B, N), dtype=np.float32)
    ub = rng.random(B, dtype=np.float32)
    m, path, bonus, committed, _ = oracle.tree_accept_sample(
        np.broadcast_to(parent, (B, N)), np.broadcast_to(tok, (B, N)), np.ascontiguousarray(logits), ua, ub,
        temperature=temperature, path_cap=4)

    def softmax(x):
        z = np.exp((x.astype(np.float64) - x.max()) / temperature)
        return z / z.sum()

    def check(samples, p, what):
        cnt = np.bincount(samples, minlength=V).astype(np.float64)
        n = cnt.sum()
        sd = np.sqrt(n * p * (1 - p)) + 1.0
        assert np.all(np.abs(cnt - n * p) <= 4.5 * sd), (what, cnt / n, p)

    check(committed[:, 0], softmax(base[0]), "first token")
    for child in (1, 2, 3):                              # went down to that child: next token ~ its distribution
        sel = path[:, 1] == child
        assert sel.sum() > 2000
        check(committed[sel, 1], softmax(base[child]), f"token after node {child}")
    sel = path[:, 2] == 4                                # two levels down
    assert sel.sum() > 500
    check(committed[sel, 2], softmax(base[4]), "token after node 4")
    # acceptance frequency of the first candidate is its target probability (point-mass proposal)
    p_first = softmax(base[0])[tok[1]]
    frac = np.mean(path[:, 1] == 1)
    assert abs(frac - p_first) < 4.5 * np.sqrt(p_first * (1 - p_first) / B)


@pytest.mark.parametrize("seed", range(6))
def test_zero_temperature_limit_is_the_greedy_walk(oracle, seed):
    """At a temperature far below the logit gaps the target distribution is a point mass on the
    argmax, so the walk must coincide with the (separately pinned) greedy acceptance."""
    rng = np.random.default_rng(500 + seed)
    B, N, V = 5, 24, 50
    parent = np.stack([W.random_tree(rng, N, max_depth=5) for _ in range(B)])
    logits = (rng.permuted(np.tile(np.arange(V, dtype=np.float32), (B, N, 1)), axis=2)) * 0.5   # gaps >= 0.5
    amax = oracle.node_argmax(logits)
    tok = np.zeros((B, N), dtype=np.int32)                   # sibling-distinct tokens, often the greedy one
    for b in range(B):
        for node in range(N):
            kids = [i for i in range(1, N) if parent[b, i] == node]
            if not kids:
                continue
            pool = [t for t in rng.permutation(V) if t != amax[b, node]][:len(kids)]
            if rng.random() < 0.6:
                pool[int(rng.integers(len(kids)))] = int(amax[b, node])
            tok[b, kids] = pool
    ua = rng.uniform(0.01, 0.99, size=(B, N)).astype(np.float32)
    ub = rng.uniform(0.01, 0.99, size=B).astype(np.float32)
    m, path, bonus, committed, _ = oracle.tree_accept_sample(parent, tok, logits, ua, ub, temperature=1e-2, path_cap=8)
    gm, gpath, gbonus, gcommitted = oracle.tree_accept(parent, tok, amax, path_cap=8)
    assert np.array_equal(m, gm) and np.array_equal(path, gpath)
    assert np.array_equal(bonus, gbonus) and np.array_equal(committed, gcommitted)
    assert m.max() >= 1


@pytest.mark.parametrize("alpha,gamma", [(0.8, 5), (0.5, 7)])
def test_chain_accept_length_follows_sigma_closed_form(oracle, alpha, gamma):
    """Chain of gamma drafted tokens, each with target probability alpha at its parent:
    E[accepted drafts] = alpha (1 - alpha^gamma) / (1 - alpha)  (Sec. 3.1)."""
    rng = np.random.default_rng(42)
    B, N, V = 200_000, gamma + 1, 4
    parent = np.arange(-1, gamma, dtype=np.int32)
    tok = np.full(N, 2, dtype=np.int32)
    rest = (1 - alpha) / (V - 1)
    p = np.full(V, rest); p[2] = alpha
    logits = np.ascontiguousarray(np.broadcast_to(log_probs(p), (B, N, V)))
    ua = rng.random((B, N), dtype=np.float32)
    ub = rng.random(B, dtype=np.float32)
    m, *_ = oracle.tree_accept_sample(np.broadcast_to(parent, (B, N)), np.broadcast_to(tok, (B, N)), logits, ua, ub,
                                      path_cap=gamma + 1)
    want = alpha * (1 - alpha ** gamma) / (1 - alpha)
    assert abs(m.mean() - want) < 4.5 * m.std() / np.sqrt(B)


def test_bad_tokens_path_cap_and_ragged_nodes(oracle):
    parent = np.array([[-1, 0, 1, 2]], dtype=np.int32)
    logits = log_probs([[0.5, 0.5]] * 4).reshape(1, 4, 2)
    ua = np.zeros((1, 4), dtype=np.float32)                   # u = 0 accepts anything with positive probability
    # out-of-range token is rejected
    m, path, *_ = oracle.tree_accept_sample(parent, [[0, 7, 0, 0]], logits, ua, [0.1], path_cap=8)
    assert m[0] == 0
    # path_cap stops the walk
    m, path, *_ = oracle.tree_accept_sample(parent, [[0, 1, 0, 1]], logits, ua, [0.1], path_cap=3)
    assert m[0] == 2 and path[0].tolist() == [0, 1, 2]
    # nodes past num_nodes do not exist
    m, path, *_ = oracle.tree_accept_sample(parent, [[0, 1, 0, 1]], logits, ua, [0.1], num_nodes=[2], path_cap=8)
    assert m[0] == 1
    with pytest.raises(ValueError):
        oracle.tree_accept_sample(np.array([[-1, 1]], dtype=np.int32), [[0, 0]], logits[:, :2], ua[:, :2], [0.1])
