"""GPU parity of specvlm_tree_verify_attn against the fp64 oracle (through the C ABI)."""
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


def run_both(sv, oracle, case, *, num_splits=0, scale=None, want_lse=True):
    from gpu_util import i32, to_dev, to_host_f64
    q, k, v = to_dev(case["q"]), to_dev(case["k"]), to_dev(case["v"])
    P, par = i32(case["prefix_len"]), i32(case["parent"])
    nn = None if case["num_nodes"] is None else i32(case["num_nodes"])
    bt = None if case["block_table"] is None else i32(case["block_table"])
    B, N, H, D = case["q"].shape
    out = torch.full_like(q, 7.0)                       # rows >= num_nodes must stay untouched
    lse = torch.full((B, H, N), 7.0, dtype=torch.float32, device="cuda") if want_lse else None
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.specvlm_tree_verify_attn(q, k, v, P, par, num_nodes=nn, block_table=bt, out=out, lse=lse,
                                err_flag=err, softmax_scale=0.0 if scale is None else scale,
                                num_splits=num_splits)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    ref_o, ref_lse = oracle.tree_attn(case["q"], case["k"], case["v"], case["prefix_len"], case["parent"],
                                      case["num_nodes"], scale=scale, block_table=case["block_table"])
    return to_host_f64(out), (None if lse is None else to_host_f64(lse)), ref_o, ref_lse


def check(case, got_o, got_lse, ref_o, ref_lse, what):
    from gpu_util import assert_attn_close, valid_rows_mask
    B, N, H, D = case["q"].shape
    rows = valid_rows_mask(B, N, case["num_nodes"])
    assert_attn_close(got_o[rows], ref_o[rows], case["dtype"], what)
    assert np.all(got_o[~rows] == 7.0), f"{what}: rows past num_nodes were written"
    if got_lse is not None:
        lrows = np.broadcast_to(rows[:, None, :], got_lse.shape)
        tol = 2e-2 if case["dtype"] == "bf16" else 1e-5
        assert np.abs(got_lse[lrows] - ref_lse[lrows]).max() <= tol, f"{what}: lse"
        assert np.all(got_lse[~lrows] == 7.0)


def test_c1_fp32_config(sv, oracle):
    """Config 1: fp32, 4 heads, D 64, prefix 64, 8-node random tree; tolerance 1e-5."""
    cfg = W.CONFIGS["C1"]
    lay = W.make_attn_layer(cfg, 0)
    tb = W.make_trees(cfg)
    case = dict(q=lay.q, k=lay.k, v=lay.v, prefix_len=lay.prefix_len, num_nodes=None,
                parent=tb.parent, block_table=None, dtype="f32")
    check(case, *run_both(sv, oracle, case), "C1")


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_cases_ragged_gqa(sv, oracle, D, dtype):
    """Several requests, ragged node counts, grouped KV heads, an empty prefix, explicit scale."""
    from gpu_util import random_case
    case = random_case(11, dtype, B=3, Hq=4, Hkv=2, D=D, N_max=20, P_list=[37, 0, 130],
                       num_nodes=[20, 1, 13])
    check(case, *run_both(sv, oracle, case, scale=0.11), f"small D={D} {dtype}")


@pytest.mark.parametrize("num_splits", [1, 2, 3, 5, 8, 9, 16])
def test_bf16_split_counts_span_tiles_and_tail(sv, oracle, num_splits):
    """S = 333+60 keys: 25 sixteen-key blocks, a ragged last block, an odd tile count;
    more splits than some ranges have blocks."""
    from gpu_util import random_case
    case = random_case(21 + num_splits, "bf16", B=2, Hq=3, Hkv=3, D=128, N_max=60, P_list=[333, 45],
                       num_nodes=[60, 33])
    check(case, *run_both(sv, oracle, case, num_splits=num_splits), f"splits={num_splits}")


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("D,num_splits", [(128, 4), (64, 6), (128, 6)])
def test_bf16_between_one_and_two_workgroups_per_compute_unit(sv, oracle, D, num_splits, paged):
    """80 (request, head) pairs x 4 or 6 splits = 320 or 480 work items: more than the chip's 256 compute
    units, at most two per unit -- the launch shape with the small rings.  Ragged lengths, an empty
    prefix, grouped KV heads, more splits than the short requests have tiles."""
    from gpu_util import random_case
    case = random_case(51 + D + num_splits, "bf16", B=5, Hq=16, Hkv=8, D=D, N_max=37,
                       P_list=[300, 0, 77, 150, 513], num_nodes=[37, 5, 20, 1, 33], paged=paged)
    check(case, *run_both(sv, oracle, case, num_splits=num_splits), f"2 per CU D={D} splits={num_splits} paged={paged}")


@pytest.mark.parametrize("D", [64, 128])
def test_bf16_paged_cache(sv, oracle, D):
    from gpu_util import random_case
    case = random_case(31, "bf16", B=3, Hq=2, Hkv=2, D=D, N_max=64, P_list=[200, 16, 95],
                       num_nodes=[64, 17, 48], paged=True)
    check(case, *run_both(sv, oracle, case, num_splits=3), f"paged D={D}")


def test_fp32_paged_cache(sv, oracle):
    from gpu_util import random_case
    case = random_case(32, "f32", B=2, Hq=2, Hkv=1, D=64, N_max=9, P_list=[40, 3], paged=True)
    check(case, *run_both(sv, oracle, case), "paged f32")


def test_bf16_chain_and_single_node(sv, oracle):
    """The oracle's two textbook special cases, on the GPU: chain tree and one-node tree."""
    from gpu_util import random_case
    case = random_case(41, "bf16", B=1, Hq=2, Hkv=2, D=128, N_max=40, P_list=[77], tree="chain")
    check(case, *run_both(sv, oracle, case), "chain")
    case = random_case(42, "bf16", B=2, Hq=2, Hkv=2, D=128, N_max=1, P_list=[77, 0])
    check(case, *run_both(sv, oracle, case), "single node")


def test_vector_alu_measurement_entry_agrees(sv, oracle):
    """The measurement aid (bf16 input through the vector-ALU kernel, no matrix cores) computes the
    same operation: within the bf16 tolerance of the oracle, contiguous and paged."""
    from gpu_util import random_case, i32, to_dev, to_host_f64
    for paged in (False, True):
        case = random_case(45, "bf16", B=2, Hq=4, Hkv=2, D=128, N_max=33, P_list=[333, 40], num_nodes=[33, 9], paged=paged)
        q, k, v = to_dev(case["q"]), to_dev(case["k"]), to_dev(case["v"])
        out = torch.full_like(q, 7.0)
        lse = torch.full((2, 4, 33), 7.0, dtype=torch.float32, device="cuda")
        err = torch.zeros(1, dtype=torch.int32, device="cuda")
        sv.specvlm_tree_verify_attn_vector_alu(q, k, v, i32(case["prefix_len"]), i32(case["parent"]), out=out, lse=lse,
                                               num_nodes=i32(case["num_nodes"]), err_flag=err,
                                               block_table=None if not paged else i32(case["block_table"]))
        torch.cuda.synchronize()
        assert int(err.item()) == 0
        ref_o, ref_lse = oracle.tree_attn(case["q"], case["k"], case["v"], case["prefix_len"], case["parent"],
                                          case["num_nodes"], block_table=case["block_table"])
        check(case, to_host_f64(out), to_host_f64(lse), ref_o, ref_lse, f"vector ALU, paged={paged}")


def test_bf16_mask_leak_detectors(sv, oracle):
    """V == 1 gives o == 1 up to one bf16 step; huge finite K/V in invisible tree slots and
    NaN beyond the request's end change nothing."""
    from gpu_util import random_case, i32, to_dev, to_host_f64
    case = random_case(51, "bf16", B=1, Hq=2, Hkv=2, D=128, N_max=24, P_list=[100])
    ones = np.full_like(case["v"], 0x3F80)              # bf16 1.0
    S = 124
    ones[:, :, S:] = W.NAN_BITS_BF16
    c1 = dict(case, v=ones)
    got, _, _, _ = run_both(sv, oracle, c1, num_splits=2)
    assert np.abs(got - 1.0).max() <= 2 ** -7
    # every query in turn: poison what it must not see
    base = run_both(sv, oracle, case, num_splits=2)[0]
    anc, _ = oracle.ancestors(case["parent"][0])
    for i in (3, 11, 23):
        k2, v2 = case["k"].copy(), case["v"].copy()
        for j in range(24):
            if not anc[i, j]:
                k2[0, :, 100 + j] = W.f32_to_bf16_bits(np.float32(30.0))
                v2[0, :, 100 + j] = W.f32_to_bf16_bits(np.float32(1e4))
        got2 = run_both(sv, oracle, dict(case, k=k2, v=v2), num_splits=2)[0]
        assert np.array_equal(got2[0, i], base[0, i])


def test_strided_q_and_out(sv, oracle):
    """q and o live inside a fused [B,N,3,H,D] projection buffer (non-dense strides)."""
    from gpu_util import random_case, i32, to_dev, to_host_f64, assert_attn_close
    case = random_case(61, "bf16", B=2, Hq=2, Hkv=2, D=128, N_max=30, P_list=[50, 64])
    fused = torch.zeros((2, 30, 3, 2, 128), dtype=torch.bfloat16, device="cuda")
    fused[:, :, 0] = to_dev(case["q"])
    outbuf = torch.zeros_like(fused)
    sv.specvlm_tree_verify_attn(fused[:, :, 0], to_dev(case["k"]), to_dev(case["v"]), i32(case["prefix_len"]),
                                i32(case["parent"]), out=outbuf[:, :, 1])
    torch.cuda.synchronize()
    ref, _ = oracle.tree_attn(case["q"], case["k"], case["v"], case["prefix_len"], case["parent"])
    assert_attn_close(to_host_f64(outbuf[:, :, 1]), ref, "bf16", "strided")
    assert float(outbuf[:, :, 0].abs().max()) == 0.0 and float(outbuf[:, :, 2].abs().max()) == 0.0


def test_error_reporting(sv):
    """Host-detectable misuse returns a status; data-dependent misuse sets the device flag."""
    from gpu_util import random_case, i32, to_dev
    case = random_case(71, "bf16", B=1, Hq=1, Hkv=1, D=128, N_max=8, P_list=[20])
    q, k, v = to_dev(case["q"]), to_dev(case["k"]), to_dev(case["v"])
    P = i32(case["prefix_len"])
    bad_parent = i32(np.array([[-1, 0, 2, 1, 0, 0, 0, 0]]))         # parent[2] = 2 is not < 2
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = torch.full_like(q, 3.0)
    sv.specvlm_tree_verify_attn(q, k, v, P, bad_parent, out=out, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) & 1
    err.zero_()
    sv.specvlm_tree_verify_attn(q, k, v, i32([k.shape[2]]), i32(case["parent"]), out=out, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) & 4                                       # prefix + nodes > capacity
    err.zero_()
    sv.specvlm_tree_verify_attn(q, k, v, P, i32(case["parent"]), num_nodes=i32([9]), out=out, err_flag=err)
    torch.cuda.synchronize()
    assert sv.err_flag_names(int(err.item())) == ["BAD_NUM_NODES"]   # more nodes than N_max
    with pytest.raises(sv.SpecvlmError, match="INVALID_ARG"):
        sv.specvlm_tree_verify_attn(q[..., :96], k[..., :96], v[..., :96], P, i32(case["parent"]))
    with pytest.raises(sv.SpecvlmError, match="INVALID_ARG"):        # the documented range of num_splits is 0 .. 64
        sv.specvlm_tree_verify_attn(q, k, v, P, i32(case["parent"]), num_splits=65)
    with pytest.raises(sv.SpecvlmError, match="WORKSPACE_TOO_SMALL"):
        sv.specvlm_tree_verify_attn(q, k, v, P, i32(case["parent"]), num_splits=4,
                                    workspace=torch.zeros(256, dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("dtype,splits", [("bf16", 1), ("bf16", 3), ("f32", 0)])
def test_block_table_entry_outside_the_pool_is_reported(sv, oracle, dtype, splits):
    """A block id outside [0, num_blocks) sets SPECVLM_ERR_BAD_BLOCK (matrix-core and vector-ALU
    kernels), nothing outside the pool is touched, and the other request's result is unharmed."""
    from gpu_util import random_case, i32, to_dev, to_host_f64, assert_attn_close
    case = random_case(75, dtype, B=2, Hq=2, Hkv=2, D=128 if dtype == "bf16" else 64, N_max=20, P_list=[150, 70], paged=True)
    nb = case["k"].shape[0]
    ref, _ = oracle.tree_attn(case["q"], case["k"], case["v"], case["prefix_len"], case["parent"],
                              block_table=case["block_table"])
    q, k, v = to_dev(case["q"]), to_dev(case["k"]), to_dev(case["v"])
    P, par = i32(case["prefix_len"]), i32(case["parent"])
    for bad in (nb, nb + 12345, -1, -(1 << 30)):
        table = case["block_table"].copy()
        table[0, 3] = bad                                            # inside request 0's prefix
        err = torch.zeros(1, dtype=torch.int32, device="cuda")
        out = sv.specvlm_tree_verify_attn(q, k, v, P, par, block_table=i32(table), err_flag=err, num_splits=splits)
        torch.cuda.synchronize()
        assert sv.err_flag_names(int(err.item())) == ["BAD_BLOCK"], bad
        assert_attn_close(to_host_f64(out)[1], ref[1], dtype, f"request 1 with a bad entry {bad} in request 0's table")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.specvlm_tree_verify_attn(q, k, v, P, par, block_table=i32(case["block_table"]), err_flag=err, num_splits=splits)
    torch.cuda.synchronize()
    assert int(err.item()) == 0


def test_one_workspace_across_shapes_and_graph_replays(sv, oracle):
    """The workspace is zero-filled once and then shared by calls of different shapes (every call
    leaves its counters zero); a captured call replays to the eager result, with eager work and
    synchronisations between the replays."""
    from gpu_util import random_case, i32, to_dev, to_host_f64, assert_attn_close
    big = random_case(81, "bf16", B=2, Hq=4, Hkv=4, D=128, N_max=60, P_list=[700, 90])
    small = random_case(82, "bf16", B=1, Hq=2, Hkv=1, D=64, N_max=17, P_list=[130])
    refs = {id(c): oracle.tree_attn(c["q"], c["k"], c["v"], c["prefix_len"], c["parent"])[0] for c in (big, small)}
    dev = {id(c): tuple(to_dev(c[x]) for x in ("q", "k", "v")) + (i32(c["prefix_len"]), i32(c["parent"]))
           for c in (big, small)}
    ws = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    for rnd in range(3):
        for c, splits in ((big, 5), (small, 3), (big, 2), (small, 7)):
            q, k, v, P, par = dev[id(c)]
            out = sv.specvlm_tree_verify_attn(q, k, v, P, par, workspace=ws, num_splits=splits)
            assert_attn_close(to_host_f64(out), refs[id(c)], "bf16", f"round {rnd} splits {splits}")
    # graph capture of one call; the inputs are refreshed in place between replays
    q, k, v, P, par = dev[id(big)]
    out = torch.zeros_like(q)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sv.specvlm_tree_verify_attn(q, k, v, P, par, out=out, workspace=ws, num_splits=4)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sv.specvlm_tree_verify_attn(q, k, v, P, par, out=out, workspace=ws, num_splits=4)
    rng = np.random.default_rng(83)
    for rep in range(3):
        q_np = W.normal(rng, big["q"].shape, 1.0, "bf16")
        q.copy_(to_dev(q_np))
        out.zero_()
        g.replay()
        torch.cuda.synchronize()
        eager = sv.specvlm_tree_verify_attn(q, k, v, P, par, workspace=ws, num_splits=4)
        assert torch.equal(out, eager), f"replay {rep}"
        ref = oracle.tree_attn(q_np, big["k"], big["v"], big["prefix_len"], big["parent"])[0]
        assert_attn_close(to_host_f64(out), ref, "bf16", f"replay {rep}")


def test_one_workspace_across_head_counts(sv, oracle):
    """Split calls with 4, 64 and 36 (request, head) pairs alternate on one workspace that was
    zero-filled once: every call must leave the counter region (a fixed 512 KiB at the start, whatever the shape) zero,
    and no call may keep partial results where another keeps counters."""
    from gpu_util import random_case, i32, to_dev, to_host_f64, assert_attn_close
    cases = [random_case(84, "bf16", B=1, Hq=4, Hkv=2, D=128, N_max=60, P_list=[400]),
             random_case(85, "bf16", B=2, Hq=32, Hkv=8, D=128, N_max=33, P_list=[150, 260]),
             random_case(86, "bf16", B=3, Hq=12, Hkv=12, D=64, N_max=64, P_list=[90, 0, 310])]
    refs = [oracle.tree_attn(c["q"], c["k"], c["v"], c["prefix_len"], c["parent"])[0] for c in cases]
    dev = [tuple(to_dev(c[x]) for x in ("q", "k", "v")) + (i32(c["prefix_len"]), i32(c["parent"])) for c in cases]
    ws = torch.zeros(1 << 24, dtype=torch.uint8, device="cuda")
    order = [(0, 8), (1, 3), (0, 5), (2, 4), (1, 8), (2, 2), (0, 3), (1, 2)]
    for rnd in range(2):
        for ci, splits in order:
            q, k, v, P, par = dev[ci]
            out = sv.specvlm_tree_verify_attn(q, k, v, P, par, workspace=ws, num_splits=splits)
            assert_attn_close(to_host_f64(out), refs[ci], "bf16", f"round {rnd} case {ci} splits {splits}")
            assert int(ws[:1024 * 4 * 128].view(torch.int32).abs().max()) == 0, "counter region not left zero"


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_sweep(sv, oracle, seed):
    """Seeded random geometry: batch, grouped heads, head size, node counts, prefix lengths from
    empty to several dozen tiles, split counts (incl. more splits than tiles), paged or contiguous."""
    from gpu_util import random_case
    rng = np.random.default_rng(9000 + seed)
    B = int(rng.integers(1, 4))
    group = int(rng.choice([1, 1, 2, 4]))
    Hkv = int(rng.choice([1, 2, 3]))
    D = int(rng.choice([64, 128]))
    N = int(rng.integers(1, 65))
    P = [int(x) for x in rng.choice([0, 1, 15, 16, 31, 33, 100, 255, 640, 1500], size=B)]
    nn = [int(rng.integers(1, N + 1)) for _ in range(B)]
    nn[0] = N
    splits = int(rng.choice([0, 1, 2, 3, 4, 7, 8, 12, 40]))
    paged = bool(rng.integers(0, 2))
    case = random_case(7000 + seed, "bf16", B=B, Hq=Hkv * group, Hkv=Hkv, D=D, N_max=N, P_list=P, num_nodes=nn,
                       paged=paged, depth=int(rng.integers(1, 8)))
    check(case, *run_both(sv, oracle, case, num_splits=splits),
          f"seed {seed}: B={B} Hq={Hkv * group} Hkv={Hkv} D={D} N={N} P={P} nn={nn} splits={splits} paged={paged}")


def test_long_video_prefix(sv, oracle):
    """A prefix of 150001 tokens (a long video): thousands of tiles per stream, ragged tail, the
    library's own split choice and the largest split count."""
    from gpu_util import random_case
    case = random_case(71, "bf16", B=1, Hq=2, Hkv=2, D=128, N_max=40, P_list=[150001])
    for splits in (0, 64):
        check(case, *run_both(sv, oracle, case, num_splits=splits), f"long prefix, splits={splits}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_requests_more_than_4_gib_apart(sv, oracle, dtype):
    """The two requests' caches sit 4.6 GB apart inside one allocation (batch stride beyond 32 bits
    in bytes, for fp32 also close to 2^31 in elements)."""
    from gpu_util import random_case, i32, to_dev, to_host_f64, assert_attn_close
    case = random_case(72, dtype, B=2, Hq=4, Hkv=2, D=128, N_max=33, P_list=[700, 129])
    B, Hkv, cap, D = case["k"].shape
    esize = 2 if dtype == "bf16" else 4
    stride_b = (4_600_000_000 // esize) // 128 * 128
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    views = []
    for name in ("k", "v"):
        big = torch.empty(stride_b + Hkv * cap * D, dtype=tdt, device="cuda")
        view = big.as_strided((B, Hkv, cap, D), (stride_b, cap * D, D, 1))
        view.copy_(to_dev(case[name]))
        views.append(view)
    out = sv.specvlm_tree_verify_attn(to_dev(case["q"]), views[0], views[1], i32(case["prefix_len"]),
                                      i32(case["parent"]))
    torch.cuda.synchronize()
    ref, _ = oracle.tree_attn(case["q"], case["k"], case["v"], case["prefix_len"], case["parent"])
    assert_attn_close(to_host_f64(out), ref, dtype, f"far-apart requests, {dtype}")


def test_paged_pool_larger_than_4_gib(sv, oracle):
    """Block ids near the end of a 5.7 GB pool: the oracle sees the same blocks renumbered densely."""
    from gpu_util import random_case, i32, to_dev, to_host_f64, assert_attn_close
    case = random_case(73, "bf16", B=2, Hq=2, Hkv=2, D=128, N_max=64, P_list=[300, 41], paged=True)
    nb_small, Hkv, bs, D = case["k"].shape
    nb_big = 700_000
    rng = np.random.default_rng(74)
    where = np.sort(rng.choice(np.arange(nb_big - 5000, nb_big), size=nb_small, replace=False))
    where[0] = 3                                         # one block near the start as well
    pools = []
    for name in ("k", "v"):
        pool = torch.empty((nb_big, Hkv, bs, D), dtype=torch.bfloat16, device="cuda")
        pool[torch.from_numpy(where).cuda()] = to_dev(case[name])
        pools.append(pool)
    table_big = where[case["block_table"]].astype(np.int32)
    out = sv.specvlm_tree_verify_attn(to_dev(case["q"]), pools[0], pools[1], i32(case["prefix_len"]),
                                      i32(case["parent"]), block_table=i32(table_big))
    torch.cuda.synchronize()
    ref, _ = oracle.tree_attn(case["q"], case["k"], case["v"], case["prefix_len"], case["parent"],
                              block_table=case["block_table"])
    assert_attn_close(to_host_f64(out), ref, "bf16", "large paged pool")


def test_two_streams_with_their_own_workspaces(sv, oracle):
    """Calls on two HIP streams overlap freely as long as each stream has its own workspace:
    20 calls per stream, issued alternately, every output equal to the same call made alone."""
    from gpu_util import random_case, i32, to_dev, to_host_f64, assert_attn_close
    cases = [random_case(81, "bf16", B=1, Hq=8, Hkv=8, D=128, N_max=60, P_list=[2000]),
             random_case(82, "bf16", B=2, Hq=4, Hkv=2, D=128, N_max=33, P_list=[700, 1300])]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    dev, alone, ws, outs = [], [], [], []
    for c in cases:
        t = dict(q=to_dev(c["q"]), k=to_dev(c["k"]), v=to_dev(c["v"]), P=i32(c["prefix_len"]), par=i32(c["parent"]))
        desc = sv.binding.make_attn_desc(t["q"], t["k"], t["q"], num_splits=8)
        t["desc"] = desc
        dev.append(t)
        ws.append(torch.zeros(sv.specvlm_tree_verify_attn_workspace_bytes(desc), dtype=torch.uint8, device="cuda"))
        alone.append(sv.specvlm_tree_verify_attn(t["q"], t["k"], t["v"], t["P"], t["par"], desc=desc).clone())
        outs.append([torch.zeros_like(t["q"]) for _ in range(20)])
    torch.cuda.synchronize()
    for it in range(20):
        for s in range(2):
            t = dev[s]
            with torch.cuda.stream(streams[s]):
                sv.specvlm_tree_verify_attn(t["q"], t["k"], t["v"], t["P"], t["par"], out=outs[s][it],
                                            workspace=ws[s], desc=t["desc"], stream=streams[s])
    torch.cuda.synchronize()
    for s in range(2):
        for it in range(20):
            assert torch.equal(outs[s][it], alone[s]), f"stream {s} call {it}"
        ref, _ = oracle.tree_attn(cases[s]["q"], cases[s]["k"], cases[s]["v"], cases[s]["prefix_len"], cases[s]["parent"])
        assert_attn_close(to_host_f64(alone[s]), ref, "bf16", f"stream {s}")


@pytest.mark.parametrize("D", [64, 128])
def test_capacity_far_above_the_lengths(sv, oracle, D):
    """A contiguous cache much longer than the requests (poisoned beyond their ends): first tiles
    that lie inside the capacity but partly or wholly past a request's last key."""
    from gpu_util import random_case
    for seed, P_list, nodes in ((91, [100, 3, 1000], [60, 5, 33]), (92, [0, 517, 31], [1, 64, 40])):
        case = random_case(seed, "bf16", B=3, Hq=4, Hkv=2, D=D, N_max=64, P_list=P_list, num_nodes=nodes,
                           cap_extra=3000)
        for splits in (0, 1, 3, 8, 16):
            check(case, *run_both(sv, oracle, case, num_splits=splits), f"seed {seed} D={D} splits={splits}")
