"""GPU parity at the five workload configurations' full sizes, in the launch configuration
bench.py times (library-chosen split count, workspace reused across layers).

Attention: element-wise against the oracle on whole layers, all heads, two layers per
configuration (three for C5: first, middle, last).  Verify step: argmax, acceptance walk and KV compaction
bit-exact against the oracle; for C5 (16 GB of cache) the oracle compacts three sampled
layers and every other layer is checked through the gather property on the device.
"""
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


def _attn_case(cfg, layer, heads=None):
    lay = W.make_attn_layer(cfg, layer, heads=heads)
    tb = W.make_trees(cfg)
    return lay, tb


@pytest.mark.parametrize("name,layers,heads", [("C2", (0, 31), None), ("C3", (0, 17), None),
                                               ("C4", (0, 9), None), ("C5", (0, 19, 39), None)])
def test_attention_full_size(sv, oracle, name, layers, heads):
    from gpu_util import assert_attn_close, i32, to_dev, to_host_f64
    cfg = W.CONFIGS[name]
    workspace = None
    for layer in layers:
        lay, tb = _attn_case(cfg, layer, heads)
        q, k, v = to_dev(lay.q), to_dev(lay.k), to_dev(lay.v)
        bt = None if lay.block_table is None else i32(lay.block_table)
        desc = sv.binding.make_attn_desc(q, k, q, block_table=bt)
        if heads is not None:            # a head sample must still use the full shape's split count
            full = sv.binding.make_attn_desc(q, k, q, block_table=bt)
            full.H_q = full.H_kv = cfg.H
            desc.num_splits = sv.specvlm_tree_verify_attn_num_splits(full)
        if workspace is None:            # one zero-filled workspace, reused by every layer like bench.py
            need = sv.specvlm_tree_verify_attn_workspace_bytes(desc)
            workspace = torch.zeros(max(need, 256), dtype=torch.uint8, device="cuda")
        err = torch.zeros(1, dtype=torch.int32, device="cuda")
        lse = torch.zeros((cfg.B, q.shape[2], cfg.N), dtype=torch.float32, device="cuda")
        out = sv.specvlm_tree_verify_attn(q, k, v, i32(lay.prefix_len), i32(tb.parent), block_table=bt,
                                          lse=lse, workspace=workspace, err_flag=err, desc=desc)
        torch.cuda.synchronize()
        assert int(err.item()) == 0
        ref_o, ref_lse = oracle.tree_attn(lay.q, lay.k, lay.v, lay.prefix_len, tb.parent,
                                          block_table=lay.block_table)
        assert_attn_close(to_host_f64(out), ref_o, cfg.dtype, f"{name} layer {layer}")
        assert np.abs(to_host_f64(lse) - ref_lse).max() <= 2e-2
    ncnt = min(1024 * 4 * 128, workspace.numel())                      # the ticket counters' fixed region
    assert int(workspace[:ncnt].view(torch.int32).abs().max().item()) == 0     # counters left at zero


def _rand_bits(rng, shape):
    return rng.integers(0, 65536, size=shape, dtype=np.uint16)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_verify_step_full_size(sv, oracle, name):
    """argmax -> accept -> compaction over all L layers, bit-exact (caches hold random bits)."""
    from gpu_util import i32, to_dev, to_host_bits
    cfg = W.CONFIGS[name]
    tb = W.make_trees(cfg)
    P = W.prefix_lengths(cfg)
    cap = cfg.depth + 1
    amax = sv.specvlm_node_argmax(to_dev(tb.logits))
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    m, path, bonus, committed = sv.specvlm_tree_accept(i32(tb.parent), i32(tb.draft_tok), amax, path_cap=cap,
                                                       err_flag=err)
    r_amax = oracle.node_argmax(tb.logits)
    r_m, r_path, r_bonus, r_comm = oracle.tree_accept(tb.parent, tb.draft_tok, r_amax, path_cap=cap)
    assert np.array_equal(amax.cpu().numpy(), r_amax)
    assert np.array_equal(m.cpu().numpy(), r_m) and np.array_equal(path.cpu().numpy(), r_path)
    assert np.array_equal(bonus.cpu().numpy(), r_bonus) and np.array_equal(committed.cpu().numpy(), r_comm)
    assert int(err.item()) == 0

    rng = np.random.default_rng(W.config_seed(cfg, 0, stream=5))
    S_cap = W.round_up(int(P.max()) + cfg.N, 16)
    shape = (cfg.L, cfg.B, cfg.H, S_cap, cfg.D)
    if cfg.dtype == "bf16":
        k, v = _rand_bits(rng, shape), _rand_bits(rng, shape)
    else:
        k = rng.standard_normal(shape).astype(np.float32)
        v = rng.standard_normal(shape).astype(np.float32)
    kd, vd = to_dev(k), to_dev(v)
    moved = torch.zeros((cfg.B, cap, 2), dtype=torch.int32, device="cuda")
    newp, _ = sv.specvlm_kv_compact(kd, vd, i32(P), path, m, moved_idx=moved)
    torch.cuda.synchronize()
    r_newp, r_moved = oracle.kv_compact(k, v, P, r_path, r_m)
    assert np.array_equal(newp.cpu().numpy(), r_newp) and np.array_equal(moved.cpu().numpy(), r_moved)
    assert np.array_equal(to_host_bits(kd), k) and np.array_equal(to_host_bits(vd), v)


def test_verify_step_c5_paged(sv, oracle):
    """C5: 40 layers x 40 heads, batch 4, paged cache (block 16).  Layer l's cache is the base
    layer's random bits XOR l, so all 16 GB differ while the host only draws one layer."""
    from gpu_util import i32, to_dev
    cfg = W.CONFIGS["C5"]
    tb = W.make_trees(cfg)
    P = W.prefix_lengths(cfg)
    cap = cfg.depth + 1
    amax = sv.specvlm_node_argmax(to_dev(tb.logits))
    m, path, bonus, committed = sv.specvlm_tree_accept(i32(tb.parent), i32(tb.draft_tok), amax, path_cap=cap)
    r_amax = oracle.node_argmax(tb.logits)
    r_m, r_path, r_bonus, r_comm = oracle.tree_accept(tb.parent, tb.draft_tok, r_amax, path_cap=cap)
    assert np.array_equal(amax.cpu().numpy(), r_amax)
    assert np.array_equal(m.cpu().numpy(), r_m) and np.array_equal(path.cpu().numpy(), r_path)
    assert np.array_equal(bonus.cpu().numpy(), r_bonus) and np.array_equal(committed.cpu().numpy(), r_comm)
    assert r_m.max() >= 3

    bs = cfg.block_size
    bpr = W.round_up(int(P.max()) + cfg.N, bs) // bs
    table, nb = W.block_table(np.random.default_rng(W.config_seed(cfg, 0, 3)), cfg.B, bpr)
    rng = np.random.default_rng(W.config_seed(cfg, 0, stream=5))
    base_k = _rand_bits(rng, (nb, cfg.H, bs, cfg.D))
    base_v = _rand_bits(rng, (nb, cfg.H, bs, cfg.D))
    layer_ids = torch.arange(cfg.L, dtype=torch.int16, device="cuda").view(cfg.L, 1, 1, 1, 1)
    bk = torch.from_numpy(base_k.view(np.int16)).cuda()
    bv = torch.from_numpy(base_v.view(np.int16)).cuda()
    kd = torch.bitwise_xor(bk.unsqueeze(0), layer_ids).view(torch.bfloat16)      # [L, nb, H, 16, D]
    vd = torch.bitwise_xor(bv.unsqueeze(0), layer_ids).view(torch.bfloat16)
    k_before, v_before = kd.clone(), vd.clone()
    tbl = i32(table)
    newp, _ = sv.specvlm_kv_compact(kd, vd, i32(P), path, m, block_table=tbl)
    torch.cuda.synchronize()
    assert np.array_equal(newp.cpu().numpy(), P + r_m + 1)

    # three layers against the oracle, byte for byte
    sample = [0, 17, cfg.L - 1]
    hk = np.stack([base_k ^ np.uint16(l) for l in sample])
    hv = np.stack([base_v ^ np.uint16(l) for l in sample])
    oracle.kv_compact(hk, hv, P, r_path, r_m, block_table=table)
    for j, l in enumerate(sample):
        assert np.array_equal(kd[l].view(torch.int16).cpu().numpy().view(np.uint16), hk[j])
        assert np.array_equal(vd[l].view(torch.int16).cpu().numpy().view(np.uint16), hv[j])

    # every layer: destination rows equal the OLD source rows, nothing else changed
    expect_k, expect_v = k_before.clone(), v_before.clone()
    for b in range(cfg.B):
        for j in range(int(r_m[b]) + 1):
            src, dst = int(P[b]) + int(r_path[b, j]), int(P[b]) + j
            sb, so = int(table[b, src // bs]), src % bs
            db, do = int(table[b, dst // bs]), dst % bs
            expect_k[:, db, :, do] = k_before[:, sb, :, so]
            expect_v[:, db, :, do] = v_before[:, sb, :, so]
    assert torch.equal(kd.view(torch.int16), expect_k.view(torch.int16))
    assert torch.equal(vd.view(torch.int16), expect_v.view(torch.int16))


def test_whole_step_graph_replay_c3(sv, oracle):
    """The step bench.py times, as it times it: one HIP graph of 32 attention layers (shared
    workspace), argmax + acceptance in one launch and the compaction, replayed three times.
    Layers 0 and 17 carry the seeded inputs and are compared with the oracle after every replay
    (attention element-wise, the walk and the compacted caches bit for bit)."""
    from gpu_util import assert_attn_close, i32, to_dev, to_host_bits, to_host_f64
    cfg = W.CONFIGS["C3"]
    tb = W.make_trees(cfg)
    P = W.prefix_lengths(cfg)
    cap = cfg.depth + 1
    sampled = (0, 17)
    lays = {l: W.make_attn_layer(cfg, l) for l in sampled}
    S_cap = lays[0].k.shape[2]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(W.config_seed(cfg, 0, stream=9))
    q = torch.randn((cfg.L, cfg.B, cfg.N, cfg.H, cfg.D), device="cuda", generator=gen).to(torch.bfloat16)
    k = torch.randn((cfg.L, cfg.B, cfg.H, S_cap, cfg.D), device="cuda", generator=gen).to(torch.bfloat16)
    v = torch.randn((cfg.L, cfg.B, cfg.H, S_cap, cfg.D), device="cuda", generator=gen).to(torch.bfloat16)
    for l in sampled:
        q[l] = to_dev(lays[l].q)
    out = torch.zeros_like(q)
    Pd, par, dtok, logits = i32(P), i32(tb.parent), i32(tb.draft_tok), to_dev(tb.logits)
    desc = sv.binding.make_attn_desc(q[0], k[0], out[0])
    workspace = torch.zeros(max(sv.specvlm_tree_verify_attn_workspace_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    counters = torch.zeros(cfg.B * sv.binding.COUNTER_STRIDE, dtype=torch.int32, device="cuda")
    amax = torch.zeros((cfg.B, cfg.N), dtype=torch.int32, device="cuda")
    acc = (torch.zeros(cfg.B, dtype=torch.int32, device="cuda"), torch.zeros((cfg.B, cap), dtype=torch.int32, device="cuda"),
           torch.zeros(cfg.B, dtype=torch.int32, device="cuda"), torch.zeros((cfg.B, cap), dtype=torch.int32, device="cuda"))
    newp = torch.zeros(cfg.B, dtype=torch.int32, device="cuda")
    moved = torch.zeros((cfg.B, cap, 2), dtype=torch.int32, device="cuda")

    def step():
        for l in range(cfg.L):
            sv.specvlm_tree_verify_attn(q[l], k[l], v[l], Pd, par, out=out[l], workspace=workspace, err_flag=err, desc=desc)
        sv.specvlm_node_argmax_accept(logits, par, dtok, counters=counters, amax=amax, err_flag=err, out=acc)
        sv.specvlm_kv_compact(k, v, Pd, acc[1], acc[0], new_prefix_len=newp, moved_idx=moved)

    def restore():
        for l in sampled:
            k[l] = to_dev(lays[l].k)
            v[l] = to_dev(lays[l].v)

    restore()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                           # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    r_amax = oracle.node_argmax(tb.logits)
    r_m, r_path, r_bonus, r_comm = oracle.tree_accept(tb.parent, tb.draft_tok, r_amax, path_cap=cap)
    refs = {}
    for l in sampled:
        ref_o, _ = oracle.tree_attn(lays[l].q, lays[l].k, lays[l].v, P, tb.parent)
        kk, vv = lays[l].k[None].copy(), lays[l].v[None].copy()
        r_newp, r_moved = oracle.kv_compact(kk, vv, P, r_path, r_m)
        refs[l] = (ref_o, kk[0], vv[0])
    for rep in range(3):
        restore()
        out.zero_()
        for t in acc:
            t.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(err.item()) == 0 and int(counters.sum().item()) == 0
        assert np.array_equal(amax.cpu().numpy(), r_amax), f"replay {rep}"
        assert np.array_equal(acc[0].cpu().numpy(), r_m) and np.array_equal(acc[1].cpu().numpy(), r_path)
        assert np.array_equal(acc[2].cpu().numpy(), r_bonus) and np.array_equal(acc[3].cpu().numpy(), r_comm)
        assert np.array_equal(newp.cpu().numpy(), r_newp) and np.array_equal(moved.cpu().numpy(), r_moved)
        for l in sampled:
            ref_o, ref_k, ref_v = refs[l]
            assert_attn_close(to_host_f64(out[l]), ref_o, "bf16", f"replay {rep} layer {l}")
            assert np.array_equal(to_host_bits(k[l]), ref_k) and np.array_equal(to_host_bits(v[l]), ref_v), f"replay {rep}"
