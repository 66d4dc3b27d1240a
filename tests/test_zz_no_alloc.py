"""GPU test of specvlm_tree_verify_attn_static: the entry point for callers that cannot allocate
(its scratch is a static device array inside the library), against specvlm_tree_verify_attn."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sv():
    import paper_2509_11815_amd as sv
    sv.load_library()
    return sv


def _device_case(case):
    from gpu_util import i32, to_dev
    return dict(q=to_dev(case["q"]), k=to_dev(case["k"]), v=to_dev(case["v"]), P=i32(case["prefix_len"]),
                par=i32(case["parent"]), nn=None if case["num_nodes"] is None else i32(case["num_nodes"]),
                bt=None if case["block_table"] is None else i32(case["block_table"]))


def test_static_scratch_matches_the_workspace_call_twice_in_a_row(sv, oracle):
    """Two calls in a row on the library's static scratch array, the second with a smaller input
    (fewer heads, fewer splits, a shorter prefix, paged): outputs and lse equal the workspace entry
    point's bit for bit and are within the bf16 tolerance of the fp64 oracle; then both once more,
    in the other order, so every call meets what another shape left behind."""
    from gpu_util import assert_attn_close, random_case, to_host_f64, valid_rows_mask
    big = random_case(301, "bf16", B=2, Hq=24, Hkv=8, D=128, N_max=60, P_list=[1900, 333], num_nodes=[60, 41])
    small = random_case(302, "bf16", B=1, Hq=4, Hkv=4, D=128, N_max=33, P_list=[210], paged=True)
    todo = [(big, 6), (small, 3), (small, 2), (big, 4)]
    dev = {id(c): _device_case(c) for c in (big, small)}
    for idx, (case, splits) in enumerate(todo):
        t = dev[id(case)]
        B, N, H, D = case["q"].shape
        desc = sv.binding.make_attn_desc(t["q"], t["k"], t["q"], block_table=t["bt"], num_splits=splits)
        assert 0 < sv.specvlm_tree_verify_attn_workspace_bytes(desc) <= (16 << 20)
        want = torch.full_like(t["q"], 5.0)
        want_lse = torch.full((B, H, N), 5.0, dtype=torch.float32, device="cuda")
        ws = torch.zeros(sv.specvlm_tree_verify_attn_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
        err = torch.zeros(1, dtype=torch.int32, device="cuda")
        sv.specvlm_tree_verify_attn(t["q"], t["k"], t["v"], t["P"], t["par"], num_nodes=t["nn"], block_table=t["bt"],
                                    out=want, lse=want_lse, workspace=ws, err_flag=err, desc=desc)
        got = torch.full_like(t["q"], 5.0)
        got_lse = torch.full_like(want_lse, 5.0)
        sv.specvlm_tree_verify_attn_static(t["q"], t["k"], t["v"], t["P"], t["par"], num_nodes=t["nn"],
                                           block_table=t["bt"], out=got, lse=got_lse, err_flag=err, desc=desc)
        torch.cuda.synchronize()
        assert int(err.item()) == 0
        assert torch.equal(got, want), f"call {idx}: output differs from the workspace entry point"
        assert torch.equal(got_lse, want_lse), f"call {idx}: lse differs"
        ref, _ = oracle.tree_attn(case["q"], case["k"], case["v"], case["prefix_len"], case["parent"],
                                  case["num_nodes"], block_table=case["block_table"])
        rows = valid_rows_mask(B, N, case["num_nodes"])
        assert_attn_close(to_host_f64(got)[rows], ref[rows], "bf16", f"call {idx}")


def test_static_scratch_rejects_shapes_beyond_its_size(sv):
    """A shape whose scratch need exceeds the static array is refused before anything is launched."""
    from gpu_util import i32
    B, H, N, D, cap = 8, 64, 64, 128, 4096
    q = torch.zeros((B, N, H, D), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((B, H, cap, D), dtype=torch.bfloat16, device="cuda")
    desc = sv.binding.make_attn_desc(q, k, q, num_splits=16)
    assert sv.specvlm_tree_verify_attn_workspace_bytes(desc) > (16 << 20)
    out = torch.full_like(q, 3.0)
    with pytest.raises(sv.SpecvlmError, match="WORKSPACE_TOO_SMALL"):
        sv.specvlm_tree_verify_attn_static(q, k, k, i32([100] * B), i32(np.tile(np.arange(-1, N - 1), (B, 1))),
                                           out=out, desc=desc)
    torch.cuda.synchronize()
    assert float(out.min()) == 3.0 and float(out.max()) == 3.0
