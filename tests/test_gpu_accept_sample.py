"""GPU parity of specvlm_tree_accept_sample (temperature > 0) against the fp64 oracle.

The walk compares uniform numbers with probabilities; the GPU evaluates those in fp32, the
oracle in fp64 (the row sums agree to about 1e-6).  The oracle reports how close each request
came to a boundary.  Requests whose accept comparisons all stay clear of their thresholds by
more than TOL must give the oracle's path, length and committed draft tokens bit for bit, and
nearly all requests must be such (all of them in the workload configurations).  A request that
is not clear of a threshold is not skipped: it must give what the oracle gives with that
request's uniform numbers moved by 4 TOL to one side or the other.  The bonus token must be the
oracle's too, unless the drawn position lies within TOL of an edge of that token's CDF
interval: then the neighbour across that edge is equally valid.  The three diagnostics the
oracle reports for this (margin_accept, margin_bonus, bonus_alt) are pinned on the CPU
(tests/test_oracle_accept_sample_pins.py).
"""
import os

import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def sv():
    import paper_2509_11815_amd as sv
    sv.load_library()
    return sv


def run_both(sv, oracle, parent, tok, logits, ua, ub, *, temperature, num_nodes=None, path_cap=8):
    from gpu_util import i32, to_dev
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = sv.specvlm_tree_accept_sample(
        i32(parent), i32(tok), to_dev(logits), torch.from_numpy(ua).cuda(), torch.from_numpy(ub).cuda(),
        temperature=temperature, num_nodes=None if num_nodes is None else i32(num_nodes), path_cap=path_cap,
        err_flag=err)
    torch.cuda.synchronize()
    ref = oracle.tree_accept_sample(parent, tok, logits, ua, ub, temperature=temperature, num_nodes=num_nodes,
                                    path_cap=path_cap)
    return [g.cpu().numpy() for g in got], ref, int(err.item())


def compare(got, ref, min_decisive, rerun=None):
    """rerun(b, shift) -> the oracle's (accept_len, path) of request b with its u_accept moved by shift."""
    m, path, bonus, committed = got
    r_m, r_path, r_bonus, r_committed, info = ref
    ok = info["margin_accept"] > TOL
    assert ok.mean() >= min_decisive, f"only {ok.mean():.3f} of the requests are clear of rounding"
    assert np.array_equal(m[ok], r_m[ok])
    assert np.array_equal(path[ok], r_path[ok])
    for b in np.nonzero(~ok)[0]:                        # within rounding of a threshold: either side of it is right
        assert rerun is not None
        sides = [(r_m[b], r_path[b].tolist())] + [rerun(b, s) for s in (4 * TOL, -4 * TOL)]
        assert (m[b], path[b].tolist()) in sides, f"request {b}: not the oracle's walk on either side of the threshold"
    near_edge = info["margin_bonus"] <= TOL
    bonus_ok = (bonus == r_bonus) | (near_edge & (bonus == info["bonus_alt"]))
    assert np.all(bonus_ok[ok])
    assert (bonus == r_bonus)[ok].mean() >= 0.9
    B, cap = committed.shape
    for b in np.nonzero(ok)[0]:
        assert committed[b, :r_m[b]].tolist() == r_committed[b, :r_m[b]].tolist()
        assert committed[b, r_m[b]] == bonus[b] and np.all(committed[b, r_m[b] + 1:] == -1)
    return ok


def test_hand_worked_fixture_on_gpu(sv, oracle):
    from test_oracle_accept_sample_pins import log_probs, read_fixture
    fx = read_fixture("accept_sample_worked.txt")
    parent = np.array([fx["parent"]] * 3, dtype=np.int32)
    tok = np.array([fx["draft_tok"]] * 3, dtype=np.int32)
    logits = np.ascontiguousarray(np.broadcast_to(log_probs(fx["probs"]).reshape(1, 6, 3), (3, 6, 3)))
    ua = np.array([fx[c + "_u_accept"] for c in "ABC"], dtype=np.float32)
    ub = np.array([fx[c + "_u_bonus"][0] for c in "ABC"], dtype=np.float32)
    got, ref, err = run_both(sv, oracle, parent, tok, logits, ua, ub, temperature=1.0, path_cap=4)
    compare(got, ref, 1.0)
    assert got[0].tolist() == [1, 2, 0] and got[2].tolist() == [2, 1, 2] and err == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("temperature", [1.0, 0.3])
def test_random_trees_small_vocab(sv, oracle, dtype, temperature):
    """Many requests, ragged node counts, a vocabulary that is not a multiple of the chunking."""
    rng = np.random.default_rng(7 + int(temperature * 10))
    B, N, V = 96, 40, 1003
    parent = np.stack([W.random_tree(rng, N, max_depth=6) for _ in range(B)])
    logits = W.normal(rng, (B, N, V), 2.0, dtype)
    amax = oracle.node_argmax(logits)
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    hit = rng.random((B, N)) < 0.7                              # many candidates carry the likeliest token
    par_c = np.clip(parent, 0, None)
    tok = np.where(hit, np.take_along_axis(amax, par_c, axis=1), tok).astype(np.int32)
    nn = rng.integers(1, N + 1, size=B).astype(np.int32)
    ua = rng.random((B, N), dtype=np.float32)
    ub = rng.random(B, dtype=np.float32)
    got, ref, err = run_both(sv, oracle, parent, tok, logits, ua, ub, temperature=temperature, num_nodes=nn)

    def rerun(b, shift):
        r = oracle.tree_accept_sample(parent[b:b + 1], tok[b:b + 1], logits[b:b + 1],
                                      np.clip(ua[b:b + 1] + np.float32(shift), 0.0, np.float32(1.0 - 2 ** -24)),
                                      ub[b:b + 1], temperature=temperature, num_nodes=nn[b:b + 1])
        return r[0][0], r[1][0].tolist()

    compare(got, ref, 0.95, rerun)
    assert err == 0
    if temperature < 1.0:
        assert ref[0].max() >= 2                                # the walk really goes down


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
@pytest.mark.parametrize("temperature", [1.0, 0.25])
def test_workload_trees_full_vocab(sv, oracle, name, temperature):
    """The verify step's own trees and logits (60 nodes, vocabulary 32000, bf16)."""
    cfg = W.CONFIGS[name]
    tb = W.make_trees(cfg)
    rng = np.random.default_rng(W.config_seed(cfg, 0, stream=9))
    ua = rng.random(tb.parent.shape, dtype=np.float32)
    ub = rng.random(cfg.B, dtype=np.float32)
    got, ref, err = run_both(sv, oracle, tb.parent, tb.draft_tok, tb.logits, ua, ub, temperature=temperature,
                             path_cap=cfg.depth + 1)
    compare(got, ref, 1.0)                              # every request of the seeded workloads is clear of its thresholds
    assert err == 0


@pytest.mark.parametrize("V,offset", [(40000, 0), (70003, 0), (32000, 3), (4096, 0)])
def test_vocabulary_sizes_and_unaligned_rows(sv, oracle, V, offset):
    """Chunks of up to 64 tokens per thread, the any-size path (V > 65536), rows off a 16-byte boundary."""
    from gpu_util import i32, to_dev
    rng = np.random.default_rng(V + offset)
    B, N = 6, 12
    parent = np.stack([W.random_tree(rng, N, max_depth=4) for _ in range(B)])
    full = W.normal(rng, (B, N, V + offset), 2.0, "bf16")
    logits = full[:, :, offset:]
    amax = oracle.node_argmax(logits)
    tok = np.take_along_axis(amax, np.clip(parent, 0, None), axis=1).astype(np.int32)   # every candidate = likeliest token
    ua = rng.random((B, N), dtype=np.float32)
    ub = rng.random(B, dtype=np.float32)
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    dev_logits = to_dev(full)[:, :, offset:]
    got = sv.specvlm_tree_accept_sample(i32(parent), i32(tok), dev_logits, torch.from_numpy(ua).cuda(),
                                        torch.from_numpy(ub).cuda(), temperature=0.2, err_flag=err)
    torch.cuda.synchronize()
    ref = oracle.tree_accept_sample(parent, tok, logits, ua, ub, temperature=0.2)
    compare([g.cpu().numpy() for g in got], ref, 0.8)
    assert int(err.item()) == 0 and ref[0].max() >= 1


def test_flags_and_limits(sv, oracle):
    from test_oracle_accept_sample_pins import log_probs
    parent = np.array([[-1, 0, 1, 2]], dtype=np.int32)
    logits = log_probs([[0.5, 0.5]] * 4).reshape(1, 4, 2)
    ua = np.zeros((1, 4), dtype=np.float32)
    ub = np.array([0.1], dtype=np.float32)
    got, ref, err = run_both(sv, oracle, parent, np.array([[0, 7, 0, 0]], dtype=np.int32), logits, ua, ub,
                             temperature=1.0)
    assert got[0][0] == 0 == ref[0][0] and err == 32                 # token outside the vocabulary
    got, ref, err = run_both(sv, oracle, parent, np.array([[0, 1, 0, 1]], dtype=np.int32), logits, ua, ub,
                             temperature=1.0, path_cap=3)
    assert got[0][0] == 2 == ref[0][0] and got[1][0].tolist() == [0, 1, 2] and err == 8   # path_cap reached
    bad = np.array([[-1, 1, 0, 0]], dtype=np.int32)
    err_t = torch.zeros(1, dtype=torch.int32, device="cuda")
    from gpu_util import i32, to_dev
    m, path, bonus, committed = sv.specvlm_tree_accept_sample(
        i32(bad), i32(np.array([[0, 1, 0, 1]])), to_dev(logits), torch.from_numpy(ua).cuda(),
        torch.from_numpy(ub).cuda(), err_flag=err_t)
    torch.cuda.synchronize()
    assert int(err_t.item()) & 1 and int(m.item()) == 0 and path[0, 0].item() == 0
    with pytest.raises(sv.SpecvlmError, match="INVALID_ARG"):
        sv.specvlm_tree_accept_sample(i32(parent), i32(parent), to_dev(logits), torch.from_numpy(ua).cuda(),
                                      torch.from_numpy(ub).cuda(), temperature=0.0)
