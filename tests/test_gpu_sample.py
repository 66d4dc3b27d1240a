"""GPU parity (bit-exact) of node_argmax, tree_accept and kv_compact against the oracle."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sv():
    import paper_2509_11815_amd as sv
    sv.load_library()
    return sv


# ------------------------------------------------------------------ argmax
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("V", [1, 7, 1000, 32000, 32003])
def test_argmax_matches_oracle(sv, oracle, dtype, V):
    from gpu_util import i32, to_dev
    rng = np.random.default_rng(V)
    B, N = 2, 9
    logits = W.normal(rng, (B, N, V), 2.0, dtype)
    nn = np.array([9, 4], dtype=np.int32)
    got = sv.specvlm_node_argmax(to_dev(logits), num_nodes=i32(nn)).cpu().numpy()
    assert np.array_equal(got, oracle.node_argmax(logits, nn))


def test_argmax_ties_signed_zero_inf(sv, oracle):
    from gpu_util import to_dev
    V = 4099
    x = np.full((1, 6, V), -1.0, dtype=np.float32)
    x[0, 0, [4000, 31, 2222]] = 3.0
    x[0, 1, :] = -np.inf
    x[0, 2, :] = -np.inf
    x[0, 2, 4098] = -1e30
    x[0, 3, :] = -0.0
    x[0, 3, 77] = 0.0
    x[0, 4, 4098] = np.inf
    x[0, 5, 1] = 2.0
    x[0, 5, 0] = 2.0
    for arr in (x, W.f32_to_bf16_bits(x)):
        got = sv.specvlm_node_argmax(to_dev(arr)).cpu().numpy()
        assert np.array_equal(got, oracle.node_argmax(arr))
        assert got[0].tolist() == [31, 0, 4098, 0, 4098, 0]


def test_argmax_unaligned_strided_rows(sv, oracle):
    """Rows that start off a 16-byte boundary (odd row stride, offset view)."""
    from gpu_util import to_dev
    rng = np.random.default_rng(3)
    big = W.normal(rng, (2, 5, 1037), 2.0, "bf16")
    dev = to_dev(big)
    view_np, view_dev = big[:, :, 3:1030], dev[:, :, 3:1030]
    got = sv.specvlm_node_argmax(view_dev).cpu().numpy()
    assert np.array_equal(got, oracle.node_argmax(view_np))


# ------------------------------------------------------------------ accept
@pytest.mark.parametrize("seed", range(4))
def test_accept_matches_oracle_random_trees(sv, oracle, seed):
    """Tiny vocabulary: equal sibling tokens and deep matches are frequent."""
    from gpu_util import i32
    rng = np.random.default_rng(300 + seed)
    B, N, V, cap = 200, 64, 3, 9
    parent = np.stack([W.random_tree(rng, N, 8) for _ in range(B)])
    tok = rng.integers(0, V, size=(B, N)).astype(np.int32)
    amax = rng.integers(0, V, size=(B, N)).astype(np.int32)
    nn = rng.integers(1, N + 1, size=B).astype(np.int32)
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = sv.specvlm_tree_accept(i32(parent), i32(tok), i32(amax), num_nodes=i32(nn), path_cap=cap, err_flag=err)
    ref = oracle.tree_accept(parent, tok, amax, nn, path_cap=cap)
    for g, r, name in zip(got, ref, ["accept_len", "path", "bonus", "committed"]):
        assert np.array_equal(g.cpu().numpy(), r), name
    assert int(err.item()) == 0
    assert ref[0].max() >= 3


def test_accept_error_flags(sv):
    from gpu_util import i32
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    m, path, bonus, committed = sv.specvlm_tree_accept(i32([[-1, 1, 0]]), i32([[0, 0, 0]]), i32([[5, 6, 7]]),
                                                       path_cap=4, err_flag=err)
    assert int(err.item()) & 1 and int(m.item()) == 0 and path[0].tolist() == [0, -1, -1, -1]
    assert int(bonus.item()) == 5 and committed[0].tolist() == [5, -1, -1, -1]
    err.zero_()
    # chain 0-1-2 fully matching but path_cap 2: only one draft node fits
    m, path, _, committed = sv.specvlm_tree_accept(i32([[-1, 0, 1]]), i32([[0, 5, 6]]), i32([[5, 6, 7]]),
                                                   path_cap=2, err_flag=err)
    assert int(err.item()) & 8 and int(m.item()) == 1 and path[0].tolist() == [0, 1]
    assert committed[0].tolist() == [5, 6]


# ------------------------------------------------------------------ compaction
@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("alias", [True, False])
def test_compact_matches_oracle(sv, oracle, dtype, D, paged, alias):
    from gpu_util import i32, to_dev, to_host_bits
    rng = np.random.default_rng(5)
    L, B, H, bs, cap = 3, 3, 2, 16, 8
    P = np.array([5, 30, 16], dtype=np.int32)
    paths = np.array([[0, 2, 3, 7, -1, -1, -1, -1], [0, 1, 2, 3, 4, 5, 6, 9], [0, -1, -1, -1, -1, -1, -1, -1]],
                     dtype=np.int32)
    m = np.array([3, 7, 0], dtype=np.int32)
    S_cap = 48
    if paged:
        table, nb = W.block_table(rng, B, S_cap // bs, spare=0.5)
        shape = (L, nb, H, bs, D)
    else:
        table = None
        shape = (L, B, H, S_cap, D)
    if dtype == "bf16":
        k = rng.integers(0, 65536, size=shape, dtype=np.uint16)
        v = rng.integers(0, 65536, size=shape, dtype=np.uint16)
    else:
        k = rng.standard_normal(shape).astype(np.float32)
        v = rng.standard_normal(shape).astype(np.float32)
    kd, vd = to_dev(k), to_dev(v)
    moved = torch.zeros((B, cap, 2), dtype=torch.int32, device="cuda")
    Pd = i32(P)
    # new_prefix_len aliasing prefix_len (two launches) or a buffer of its own (one launch)
    newp, _ = sv.specvlm_kv_compact(kd, vd, Pd, i32(paths), i32(m), block_table=None if table is None else i32(table),
                                    new_prefix_len=Pd if alias else None, moved_idx=moved)
    torch.cuda.synchronize()
    if not alias:
        assert np.array_equal(Pd.cpu().numpy(), P)
    ref_newp, ref_moved = oracle.kv_compact(k, v, P, paths, m, block_table=table)
    assert np.array_equal(newp.cpu().numpy(), ref_newp)
    assert np.array_equal(moved.cpu().numpy(), ref_moved)
    assert np.array_equal(to_host_bits(kd), k) and np.array_equal(to_host_bits(vd), v)


def test_compact_skips_moves_through_a_bad_block_id(sv, oracle):
    """Paged cache with block ids outside the pool in one request's table: SPECVLM_ERR_BAD_BLOCK is
    set, the moves that would touch such a block are not made (nothing is written into a block the
    table does not validly name), every other move is the oracle's."""
    from gpu_util import i32, to_dev, to_host_bits
    rng = np.random.default_rng(7)
    L, B, H, bs, D = 2, 2, 2, 16, 128
    P = np.array([10, 29], dtype=np.int32)                       # both requests' paths straddle two blocks
    paths = np.array([[0, 2, 5, 9], [0, 2, 4, 6]], dtype=np.int32)
    m = np.array([3, 3], dtype=np.int32)
    table, nb = W.block_table(rng, B, 3, spare=0.5)
    k = rng.integers(0, 65536, size=(L, nb, H, bs, D), dtype=np.uint16)
    v = rng.integers(0, 65536, size=(L, nb, H, bs, D), dtype=np.uint16)
    for bad in (nb, -3):
        bad_table = table.copy()
        bad_table[0, 1] = bad                                    # request 0: slots 16..31 are unreachable
        kd, vd = to_dev(k), to_dev(v)
        err = torch.zeros(1, dtype=torch.int32, device="cuda")
        sv.specvlm_kv_compact(kd, vd, i32(P), i32(paths), i32(m), block_table=i32(bad_table), err_flag=err)
        torch.cuda.synchronize()
        assert sv.err_flag_names(int(err.item())) == ["BAD_BLOCK"]
        # expected: request 1 as the oracle moves it; of request 0 the two moves inside block 0
        # (slots 11 <- 12, 12 <- 15), not the one whose source, slot 19, lies in the unreachable block
        ke, ve = k.copy(), v.copy()
        valid = np.array([[0, 2, 5, -1], paths[1]], dtype=np.int32)
        oracle.kv_compact(ke, ve, P, valid, np.array([2, 3], dtype=np.int32), block_table=table)
        assert np.array_equal(to_host_bits(kd), ke) and np.array_equal(to_host_bits(vd), ve)
    kd, vd = to_dev(k), to_dev(v)
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.specvlm_kv_compact(kd, vd, i32(P), i32(paths), i32(m), block_table=i32(table), err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    oracle.kv_compact(k, v, P, paths, m, block_table=table)
    assert np.array_equal(to_host_bits(kd), k) and np.array_equal(to_host_bits(vd), v)


def test_compact_layer_pointer_array(sv, oracle):
    """Layers allocated separately and passed as a device array of pointers."""
    from gpu_util import i32, to_dev, to_host_bits
    rng = np.random.default_rng(6)
    L, B, H, S_cap, D = 4, 2, 3, 40, 128
    ks = [rng.integers(0, 65536, size=(B, H, S_cap, D), dtype=np.uint16) for _ in range(L)]
    vs = [rng.integers(0, 65536, size=(B, H, S_cap, D), dtype=np.uint16) for _ in range(L)]
    kd, vd = [to_dev(x) for x in ks], [to_dev(x) for x in vs]
    kp = torch.tensor([t.data_ptr() for t in kd], dtype=torch.int64, device="cuda")
    vp = torch.tensor([t.data_ptr() for t in vd], dtype=torch.int64, device="cuda")
    P, paths, m = np.array([7, 20], dtype=np.int32), np.array([[0, 3, 4, 9], [0, 2, -1, -1]], dtype=np.int32), np.array([3, 1], dtype=np.int32)
    newp, _ = sv.specvlm_kv_compact(kd[0], vd[0], i32(P), i32(paths), i32(m), layer_ptrs=(kp, vp))
    torch.cuda.synchronize()
    kh, vh = np.stack(ks), np.stack(vs)
    ref_newp, _ = oracle.kv_compact(kh, vh, P, paths, m)
    assert np.array_equal(newp.cpu().numpy(), ref_newp)
    for l in range(L):
        assert np.array_equal(to_host_bits(kd[l]), kh[l]) and np.array_equal(to_host_bits(vd[l]), vh[l])



# ------------------------------------------------------------------ argmax + accept in one launch
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_fused_argmax_accept_matches_oracle(sv, oracle, dtype):
    """Same results as the two separate calls; the counters are zeroed once and reused by every call."""
    from gpu_util import i32, to_dev
    rng = np.random.default_rng(17)
    B, N, V, cap = 5, 60, 1000, 8
    counters = torch.zeros(B * sv.binding.COUNTER_STRIDE, dtype=torch.int32, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    for rep in range(3):
        trees = [W.eagle_tree(rng, N, 6, 10) for _ in range(B)]
        parent = np.stack([t[0] for t in trees])
        logits, top = W.planted_logits(rng, B * N, V, 2.0, "bf16" if dtype == "bf16" else "fp32")
        logits, top = logits.reshape(B, N, V), top.reshape(B, N)
        tok = np.stack([W.draft_tokens_topk(rng, trees[b][0], trees[b][2], top[b], V, 0.8) for b in range(B)])
        nn = rng.integers(1, N + 1, size=B).astype(np.int32)
        nn[0] = N
        amax, m, path, bonus, committed = sv.specvlm_node_argmax_accept(
            to_dev(logits), i32(parent), i32(tok), num_nodes=i32(nn), path_cap=cap, counters=counters, err_flag=err)
        r_amax = oracle.node_argmax(logits, nn)
        r_m, r_path, r_bonus, r_comm = oracle.tree_accept(parent, tok, r_amax, nn, path_cap=cap)
        assert np.array_equal(amax.cpu().numpy(), r_amax)
        assert np.array_equal(m.cpu().numpy(), r_m) and np.array_equal(path.cpu().numpy(), r_path)
        assert np.array_equal(bonus.cpu().numpy(), r_bonus) and np.array_equal(committed.cpu().numpy(), r_comm)
        assert int(err.item()) == 0 and int(counters.abs().sum().item()) == 0
        assert r_m.max() >= 1 or rep < 2
    # a malformed tree: the root is committed, the flag is set, the counters are back to zero
    bad = parent.copy()
    bad[1, 2] = 2
    _, m, path, _, _ = sv.specvlm_node_argmax_accept(to_dev(logits), i32(bad), i32(tok), path_cap=cap,
                                                     counters=counters, err_flag=err)
    assert int(err.item()) & 1 and int(m[1].item()) == 0 and path[1].tolist() == [0] + [-1] * (cap - 1)
    assert int(counters.abs().sum().item()) == 0
    # one counter per request, each on a cache line of its own: a [B] tensor is too small and is refused
    with pytest.raises(ValueError):
        sv.specvlm_node_argmax_accept(to_dev(logits), i32(parent), i32(tok), path_cap=cap,
                                      counters=torch.zeros(B, dtype=torch.int32, device="cuda"), err_flag=err)


# ------------------------------------------------------------------ offsets that need 64 bits
def test_argmax_and_compact_more_than_4_gib_apart(sv, oracle):
    """Requests 4.6 GB apart in the logits; layers 4.4 GB and requests 2.3 GB apart in the caches."""
    from gpu_util import i32, to_dev, to_host_bits
    rng = np.random.default_rng(8)
    B, N, V = 2, 5, 3001
    lg = W.normal(rng, (B, N, V), 2.0, "bf16")
    stride_b = 2_300_000_000
    big = torch.empty(stride_b + N * V, dtype=torch.bfloat16, device="cuda")
    view = big.as_strided((B, N, V), (stride_b, V, 1))
    view.copy_(to_dev(lg))
    assert np.array_equal(sv.specvlm_node_argmax(view).cpu().numpy(), oracle.node_argmax(lg))
    del big, view

    L, H, S_cap, D = 2, 2, 40, 128
    k = rng.integers(0, 65536, size=(L, B, H, S_cap, D), dtype=np.uint16)
    v = rng.integers(0, 65536, size=(L, B, H, S_cap, D), dtype=np.uint16)
    sl, sb = 2_200_000_000, 1_150_000_000                  # elements
    strides = (sl, sb, S_cap * D, D, 1)
    bufs = []
    for a in (k, v):
        buf = torch.empty(sl + sb + H * S_cap * D, dtype=torch.bfloat16, device="cuda")
        t = buf.as_strided(a.shape, strides)
        t.copy_(to_dev(a))
        bufs.append(t)
    P = np.array([7, 20], dtype=np.int32)
    paths = np.array([[0, 3, 4, 9], [0, 2, -1, -1]], dtype=np.int32)
    m = np.array([3, 1], dtype=np.int32)
    newp, _ = sv.specvlm_kv_compact(bufs[0], bufs[1], i32(P), i32(paths), i32(m))
    torch.cuda.synchronize()
    ref_newp, _ = oracle.kv_compact(k, v, P, paths, m)
    assert np.array_equal(newp.cpu().numpy(), ref_newp)
    assert np.array_equal(to_host_bits(bufs[0].contiguous()), k)
    assert np.array_equal(to_host_bits(bufs[1].contiguous()), v)
