"""GPU parity of the draft-side tree growth (specvlm_draft_topk / _select / _finalize) against the oracle.

Tokens, candidate choices and the final tree are integer decisions and must match bit for bit.
A candidate's score is fp32 on the GPU (cum + (logit - lse), lse = max + log(sum exp)) and fp64
rounded once to fp32 in the oracle: both carry a few fp32 roundings of numbers of magnitude
<= ~30, so scores agree to 2e-5; a choice between two candidates whose oracle scores are
closer than 1e-4 may fall either way, the oracle reports that margin and only requests clear
of it are compared through the whole growth (every kernel is also compared on its own with
inputs that the oracle or the generator fixes).
"""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu

SCORE_TOL = 2e-5
CLEAR = 1e-4


@pytest.fixture(scope="module")
def sv():
    import paper_2509_11815_amd as sv
    sv.load_library()
    return sv


def _f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V,K", [(5, 5), (1000, 10), (32000, 10), (32003, 7), (40000, 10), (70001, 3)])
def test_topk_matches_oracle(sv, oracle, dtype, V, K):
    """Register paths (32 and 64 entries per thread, vector and scalar loads) and the any-size path."""
    from gpu_util import i32, to_dev
    rng = np.random.default_rng(V * 7 + K)
    B, Wd = 2, 3
    logits = W.normal(rng, (B, Wd, V), 2.0, dtype)
    cum = (-rng.random((B, Wd)) * 9).astype(np.float32)
    par = rng.integers(0, 500, size=(B, Wd)).astype(np.int32)
    lse = torch.empty((B, Wd), dtype=torch.float32, device="cuda")
    score, token, parent = sv.specvlm_draft_topk(to_dev(logits), K, cum=_f32(cum), parent_idx=i32(par), lse_out=lse)
    r_score, r_token, r_lse = oracle.topk_logprob(logits.reshape(B * Wd, V), K, cum.reshape(-1).astype(np.float64))
    assert np.array_equal(token.cpu().numpy().reshape(B * Wd, K), r_token)
    np.testing.assert_allclose(score.cpu().numpy().reshape(B * Wd, K), r_score, rtol=0, atol=SCORE_TOL)
    np.testing.assert_allclose(lse.cpu().numpy().reshape(-1), r_lse, rtol=0, atol=SCORE_TOL)
    assert np.array_equal(parent.cpu().numpy(), np.repeat(par, K, axis=1))


def test_topk_ties_signed_zero_inf_and_views(sv, oracle):
    from gpu_util import to_dev
    V, K = 4099, 6
    x = np.full((1, 4, V), -1.0, dtype=np.float32)
    x[0, 0, [4000, 31, 2222, 5, 4098]] = 3.0             # five equal maxima, then the lowest of the rest
    x[0, 1, :] = -0.0
    x[0, 1, [77, 1500]] = 0.0                             # -0 == +0: tokens 0..5
    x[0, 2, :] = -np.inf
    x[0, 2, [9, 4]] = [1.0, 2.0]                          # two finite values, then -inf entries in index order
    x[0, 3, 4098] = 50.0
    for arr in (x, W.f32_to_bf16_bits(x)):
        _, token, _ = sv.specvlm_draft_topk(to_dev(arr), K)
        _, r_token, _ = oracle.topk_logprob(arr.reshape(4, V), K)
        got = token.cpu().numpy().reshape(4, K)
        assert np.array_equal(got, r_token)
        assert got[0].tolist() == [5, 31, 2222, 4000, 4098, 0] and got[1].tolist() == [0, 1, 2, 3, 4, 5]
        assert got[2].tolist() == [4, 9, 0, 1, 2, 3]
    # rows off a 16-byte boundary, outputs written into a wider candidate array at an offset
    rng = np.random.default_rng(5)
    big = W.normal(rng, (2, 3, 1037), 2.0, "bf16")
    dev = to_dev(big)
    score_all = torch.full((2, 100), 7.0, dtype=torch.float32, device="cuda")
    token_all = torch.full((2, 100), -7, dtype=torch.int32, device="cuda")
    sv.specvlm_draft_topk(dev[:, :, 3:1030], 10, score_out=score_all[:, 20:50], token_out=token_all[:, 20:50])
    r_score, r_token, _ = oracle.topk_logprob(np.ascontiguousarray(big[:, :, 3:1030]).reshape(6, 1027), 10)
    assert np.array_equal(token_all[:, 20:50].cpu().numpy().reshape(6, 10), r_token)
    np.testing.assert_allclose(score_all[:, 20:50].cpu().numpy().reshape(6, 10), r_score, rtol=0, atol=SCORE_TOL)
    assert torch.all(token_all[:, :20] == -7) and torch.all(token_all[:, 50:] == -7)
    assert torch.all(score_all[:, :20] == 7.0) and torch.all(score_all[:, 50:] == 7.0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V,K", [(32000, 10), (40000, 64), (70001, 12), (900, 64)])
def test_topk_when_the_best_tokens_are_neighbours(sv, oracle, dtype, V, K):
    """Logits that rise or fall along the vocabulary, or are all equal: far more entries reach the
    kernel's first threshold than it keeps, so its any-input path has to give the same answer."""
    from gpu_util import to_dev
    ramp = np.linspace(-8.0, 8.0, V).astype(np.float32)
    x = np.stack([ramp, ramp[::-1], np.full(V, 1.5, np.float32), np.round(ramp * 4) / 4])[None]   # [1,4,V]
    arr = x if dtype == "f32" else W.f32_to_bf16_bits(x)
    score, token, _ = sv.specvlm_draft_topk(to_dev(arr), K)
    r_score, r_token, _ = oracle.topk_logprob(arr.reshape(4, V), K)
    assert np.array_equal(token.cpu().numpy().reshape(4, K), r_token)
    np.testing.assert_allclose(score.cpu().numpy().reshape(4, K), r_score, rtol=0, atol=SCORE_TOL)
    assert r_token[2].tolist() == list(range(K))                          # all equal: the lowest tokens


@pytest.mark.parametrize("C,M", [(1, 1), (10, 10), (100, 10), (610, 59), (1500, 64), (8192, 40), (256, 64), (1024, 64),
                                 (1023, 1), (700, 33), (1024, 65)])
def test_select_matches_oracle(sv, oracle, C, M):
    from gpu_util import i32
    rng = np.random.default_rng(C + M)
    B = 5
    score = (np.round(rng.normal(0, 1, size=(B, C)) * 8) / 8).astype(np.float32)       # many exact ties
    score[0, : C // 2] = -np.inf
    num = rng.integers(0, C + 1, size=B).astype(np.int32)
    num[0], num[1] = C, min(C, 3)
    sel, sel_score, count = sv.specvlm_draft_select(_f32(score), M, num_cand=i32(num), index_base=1000)
    r_sel, r_count, _ = oracle.tree_select(score, M, num)
    want = np.where(r_sel >= 0, r_sel + 1000, -1)
    assert np.array_equal(sel.cpu().numpy(), want)
    assert np.array_equal(count.cpu().numpy(), r_count)
    got_sc = sel_score.cpu().numpy()
    for b in range(B):
        assert np.array_equal(got_sc[b, :r_count[b]], score[b, r_sel[b, :r_count[b]]])
        assert np.all(got_sc[b, r_count[b]:] == -np.inf)
    # a view into a wider array, no candidate counts
    wide = _f32(np.concatenate([np.zeros((B, 7), np.float32), score], axis=1))
    sel2, _, _ = sv.specvlm_draft_select(wide[:, 7:], M)
    r2, _, _ = oracle.tree_select(score, M)
    assert np.array_equal(sel2.cpu().numpy(), r2)


@pytest.mark.parametrize("C,M", [(1024, 64), (510, 59), (777, 20)])
def test_select_when_the_winners_crowd_together(sv, oracle, C, M):
    """Score patterns that are hard on a selection which first discards by a threshold: all scores equal
    (the index decides everything), sorted either way, and every high score in candidates i with
    i mod 128 < M (whole residue classes high, so a threshold from class maxima discards the least)."""
    i = np.arange(C)
    rng = np.random.default_rng(C * 7 + M)
    rows = [np.zeros(C), -i.astype(np.float64), i.astype(np.float64), np.where(i % 128 < M, 5.0, -5.0),
            np.where(i % 128 < M, 5.0 + (i // 128), -5.0), np.where(i % 128 < M, rng.normal(5, 1, C), rng.normal(-5, 1, C)),
            np.where(i % 128 == 3, 1.0, 0.0), np.full(C, -np.inf)]
    score = np.stack(rows).astype(np.float32)
    sel, sel_score, count = sv.specvlm_draft_select(_f32(score), M)
    r_sel, r_count, _ = oracle.tree_select(score, M)
    assert np.array_equal(sel.cpu().numpy(), r_sel)
    assert np.array_equal(count.cpu().numpy(), r_count)
    got_sc = sel_score.cpu().numpy()
    for b in range(len(rows)):
        assert np.array_equal(got_sc[b, :r_count[b]], score[b, r_sel[b, :r_count[b]]])


@pytest.mark.parametrize("dtype,V", [("bf16", 32000), ("f32", 1000), ("bf16", 40000), ("bf16", 70001)])
def test_topk_select_in_one_launch_equals_the_two_calls(sv, oracle, dtype, V):
    """Same arithmetic in both: every output must be identical, with exact score ties between rows
    (two rows share their logits and cumulated scores), M above and below the candidate count,
    and twice in a row on the same counters."""
    from gpu_util import i32, to_dev
    rng = np.random.default_rng(V + 5)
    B, Wd, K = 3, 7, 10
    logits = W.normal(rng, (B, Wd, V), 2.0, dtype)
    logits[:, 4] = logits[:, 1]
    logits[:, 6] = np.sort(logits[:, 6], axis=-1)       # best tokens are neighbours: the K-rounds path
    cum = (-rng.random((B, Wd)) * 3).astype(np.float32)
    cum[:, 4] = cum[:, 1]
    par = rng.integers(0, 500, size=(B, Wd)).astype(np.int32)
    counters = torch.zeros(B * sv.binding.COUNTER_STRIDE, dtype=torch.int32, device="cuda")
    lg, cm, pr = to_dev(logits), _f32(cum), i32(par)
    score, token, parent = sv.specvlm_draft_topk(lg, K, cum=cm, parent_idx=pr)
    for M in (10, 100):
        sel, sel_score, count = sv.specvlm_draft_select(score, M, index_base=40)
        f = sv.specvlm_draft_topk_select(lg, K, M, cum=cm, parent_idx=pr, index_base=40, counters=counters)
        torch.cuda.synchronize()
        assert torch.equal(f[0], score) and torch.equal(f[1], token) and torch.equal(f[2], parent)
        assert torch.equal(f[3], sel) and torch.equal(f[4], sel_score) and torch.equal(f[5], count)
        assert int(counters.sum().item()) == 0
    # and against the oracle's selection of the oracle's own scores where the choice is clear
    r_score, _, _ = oracle.topk_logprob(logits.reshape(B * Wd, V), K, cum.reshape(-1).astype(np.float64))
    r_sel, r_count, r_gap = oracle.tree_select(r_score.reshape(B, Wd * K).astype(np.float32), 10)
    sel10 = sv.specvlm_draft_topk_select(lg, K, 10, cum=cm, parent_idx=pr, counters=counters)[3].cpu().numpy()
    for b in range(B):
        if r_gap[b] > CLEAR or r_gap[b] == 0:
            assert np.array_equal(sel10[b], r_sel[b])


def _level_logits(rng, B, V, K, width, depth, dtype):
    return [W.normal(rng, (B, 1 if d == 0 else min(width, K if d == 1 else width * K), V), 2.0, dtype)
            for d in range(depth)]


def _grow_on_gpu(sv, level_logits, root_token, K, width, N_max, fused=False):
    """The caller's loop: one select + topk per level, writing into the request's candidate arrays.
    fused: the selection for the next level is made by the level's own launch."""
    from gpu_util import i32, to_dev
    B = level_logits[0].shape[0]
    C = sum(lg.shape[1] * K for lg in level_logits)
    score = torch.zeros((B, C), dtype=torch.float32, device="cuda")
    token = torch.zeros((B, C), dtype=torch.int32, device="cuda")
    parent = torch.full((B, C), -1, dtype=torch.int32, device="cuda")
    base, count, sels = 0, 0, []
    counters = torch.zeros(B * sv.binding.COUNTER_STRIDE, dtype=torch.int32, device="cuda")
    sel = sel_score = None
    for d, lg in enumerate(level_logits):
        rows = lg.shape[1]
        new_base = base + count
        out = dict(score_out=score[:, new_base:new_base + rows * K], token_out=token[:, new_base:new_base + rows * K],
                   parent_out=parent[:, new_base:new_base + rows * K])
        if d > 0 and not fused:
            sel, sel_score, _ = sv.specvlm_draft_select(score[:, base:base + count], rows, index_base=base)
        if d > 0:
            sels.append(sel.cpu().numpy())
        if fused and d + 1 < len(level_logits):
            nxt = level_logits[d + 1].shape[1]
            res = sv.specvlm_draft_topk_select(to_dev(lg), K, nxt, cum=sel_score, parent_idx=sel, index_base=new_base,
                                               counters=counters, **out)
            sel, sel_score = res[3], res[4]
        else:
            sv.specvlm_draft_topk(to_dev(lg), K, cum=sel_score, parent_idx=sel, **out)
        base, count = new_base, rows * K
    assert int(counters.sum().item()) == 0
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    par, tok, node_cand, num_nodes = sv.specvlm_draft_finalize(score, parent, token, i32(root_token), N_max, err_flag=err)
    assert int(err.item()) == 0
    return dict(cand_score=score.cpu().numpy(), cand_token=token.cpu().numpy(), cand_parent=parent.cpu().numpy(),
                level_sel=sels, parent=par.cpu().numpy(), draft_tok=tok.cpu().numpy(),
                node_cand=node_cand.cpu().numpy(), num_nodes=num_nodes.cpu().numpy())


@pytest.mark.parametrize("name,B,V,K,width,depth,N_max,dtype", [
    ("paper", 1, 32000, 10, 10, 7, 60, "bf16"),        # Sec. 4.1: Top-K 10, 60 tokens, depth 7, batch 1
    ("batch8-depth6", 8, 32000, 10, 10, 6, 60, "bf16"),
    ("batch4-61-nodes", 4, 32000, 10, 10, 7, 61, "bf16"),
    ("small-f32", 3, 1000, 4, 6, 5, 24, "f32"),
    ("wide", 2, 5000, 8, 20, 4, 64, "bf16"),
])
@pytest.mark.parametrize("fused", [False, True])
def test_whole_growth_matches_oracle(sv, oracle, name, B, V, K, width, depth, N_max, dtype, fused):
    rng = np.random.default_rng(W.config_seed(W.CONFIGS["C3"], 0, 7) + B * 131 + V)
    lv = _level_logits(rng, B, V, K, width, depth, dtype)
    root = rng.integers(0, V, size=B).astype(np.int32)
    ref = oracle.grow_tree(lv, root, K=K, width=width, N_max=N_max)
    got = _grow_on_gpu(sv, lv, root, K, width, N_max, fused=fused)
    gaps = np.stack(ref["level_gap"] + [ref["final_gap"]])             # [levels+1, B]
    # an exact tie (margin 0: equal logits under one parent give equal scores on both sides) is
    # decided by the index rule; only a small non-zero margin is ambiguous
    clear = np.all((gaps > CLEAR) | (gaps == 0), axis=0)
    assert clear.mean() >= 0.75, gaps
    for b in np.nonzero(clear)[0]:
        assert np.array_equal(got["cand_token"][b], ref["cand_token"][b]), (name, b)
        assert np.array_equal(got["cand_parent"][b], ref["cand_parent"][b]), (name, b)
        np.testing.assert_allclose(got["cand_score"][b], ref["cand_score"][b], rtol=0, atol=SCORE_TOL)
        for g, r in zip(got["level_sel"], ref["level_sel"]):
            assert np.array_equal(g[b], r[b])
        for key in ("parent", "draft_tok", "node_cand", "num_nodes"):
            assert np.array_equal(got[key][b], ref[key][b]), (name, b, key)
    # every request, clear or not: a well-formed tree that the verification calls accept
    for b in range(B):
        par, n = got["parent"][b], int(got["num_nodes"][b])
        assert n == N_max and par[0] == -1 and np.all((par[1:n] >= 0) & (par[1:n] < np.arange(1, n)))
        assert got["draft_tok"][b, 0] == root[b] and W.tree_depths(par[:n]).max() <= depth


def test_finalize_from_oracle_candidates_and_error_bits(sv, oracle):
    """The kernel alone, on candidate arrays the oracle produced; then malformed inputs."""
    from gpu_util import i32
    rng = np.random.default_rng(77)
    B, V, K, width, depth, N_max = 6, 3000, 10, 10, 7, 60
    lv = _level_logits(rng, B, V, K, width, depth, "bf16")
    root = np.arange(B, dtype=np.int32)
    ref = oracle.grow_tree(lv, root, K=K, width=width, N_max=N_max)
    C = ref["cand_score"].shape[1]
    num = np.array([C, C, 300, 59, 10, 0], dtype=np.int32)              # ragged candidate counts
    want = oracle.tree_finalize(ref["cand_score"], ref["cand_parent"], ref["cand_token"], root, N_max, num)
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = sv.specvlm_draft_finalize(_f32(ref["cand_score"]), i32(ref["cand_parent"]), i32(ref["cand_token"]), i32(root),
                                    N_max, num_cand=i32(num), err_flag=err)
    assert int(err.item()) == 0
    for g, r in zip(got, want[:4]):
        assert np.array_equal(g.cpu().numpy(), r)
    # a child chosen without its parent, and a parent that does not precede its child
    score = _f32([[-1.0, -2.0, -0.5], [-1.0, -2.0, -0.5]])
    tok = i32([[4, 5, 6], [4, 5, 6]])
    sv.specvlm_draft_finalize(score, i32([[-1, -1, 1], [-1, 0, 0]]), tok, i32([0, 0]), 3, err_flag=err)
    assert int(err.item()) == 64
    err.zero_()
    sv.specvlm_draft_finalize(score, i32([[-1, 2, 0], [-1, 0, 0]]), tok, i32([0, 0]), 4, err_flag=err)
    assert int(err.item()) == 1
    err.zero_()
    out = sv.specvlm_draft_finalize(score, i32([[-1, 0, 0], [-1, 0, 1]]), tok, i32([7, 8]), 1, err_flag=err)   # root only
    assert int(err.item()) == 0 and out[0].cpu().numpy().tolist() == [[-1], [-1]]
    assert out[1].cpu().numpy().tolist() == [[7], [8]] and out[3].cpu().numpy().tolist() == [1, 1]


def test_grown_tree_feeds_the_verification_calls(sv, oracle):
    """Draft growth -> greedy verification of the grown tree, end to end on the GPU, against the
    oracle's growth -> oracle's verification (a request whose growth margins are clear)."""
    from gpu_util import i32, to_dev
    rng = np.random.default_rng(2024)
    B, V, K, width, depth, N_max = 2, 32000, 10, 10, 6, 60
    lv = _level_logits(rng, B, V, K, width, depth, "bf16")
    root = np.array([11, 12], dtype=np.int32)
    ref = oracle.grow_tree(lv, root, K=K, width=width, N_max=N_max)
    got = _grow_on_gpu(sv, lv, root, K, width, N_max)
    gaps = np.stack(ref["level_gap"] + [ref["final_gap"]])
    clear = np.all((gaps > CLEAR) | (gaps == 0), axis=0)
    # target logits whose greedy token follows the draft's first choice along a path of the tree
    tlog = W.normal(rng, (B, N_max, V), 2.0, "bf16")
    big = W.f32_to_bf16_bits(np.array([30.0], dtype=np.float32))[0]
    for b in range(B):
        node = 0
        for _ in range(3):
            kids = np.nonzero(ref["parent"][b] == node)[0]
            if len(kids) == 0:
                break
            tlog[b, node, ref["draft_tok"][b, kids[0]]] = big
            node = kids[0]
    amax = sv.specvlm_node_argmax(to_dev(tlog))
    m, path, bonus, committed = sv.specvlm_tree_accept(i32(got["parent"]), i32(got["draft_tok"]), amax, path_cap=depth + 1)
    r_amax = oracle.node_argmax(tlog)
    r_m, r_path, r_bonus, r_comm = oracle.tree_accept(ref["parent"], ref["draft_tok"], r_amax, path_cap=depth + 1)
    for b in np.nonzero(clear)[0]:
        assert m[b].item() == r_m[b] >= 1
        assert np.array_equal(path[b].cpu().numpy(), r_path[b]) and bonus[b].item() == r_bonus[b]
        assert np.array_equal(committed[b].cpu().numpy(), r_comm[b])
    assert clear.any()
