"""The C-ABI library loads without a GPU and exports every symbol include/specvlm.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "specvlm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(specvlm_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2509_11815_amd import build
    if build.needs_build():
        build.build()
    lib = ctypes.CDLL(build.LIB)
    names = declared_symbols()
    assert {"specvlm_tree_verify_attn", "specvlm_node_argmax", "specvlm_tree_accept",
            "specvlm_kv_compact"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    lib.specvlm_version.restype = ctypes.c_int32
    assert lib.specvlm_version() >= 100


def test_host_side_argument_checks_need_no_gpu():
    """Scalar validation happens before any HIP call."""
    import paper_2509_11815_amd as sv
    from paper_2509_11815_amd.binding import AttnDesc
    lib = sv.load_library()
    d = AttnDesc()
    assert lib.specvlm_tree_verify_attn_workspace_bytes(ctypes.byref(d)) == 0          # all-zero desc
    d.dtype, d.B, d.H_q, d.H_kv, d.D, d.N_max = 0, 1, 32, 32, 128, 60
    d.kv_capacity = 3328
    d.q_stride_b, d.q_stride_n, d.q_stride_h = 60 * 32 * 128, 32 * 128, 128
    d.o_stride_b, d.o_stride_n, d.o_stride_h = 60 * 32 * 128, 32 * 128, 128
    d.kv_stride_b, d.kv_stride_h, d.kv_stride_t = 32 * 3328 * 128, 3328 * 128, 128
    need = lib.specvlm_tree_verify_attn_workspace_bytes(ctypes.byref(d))
    assert need > 0
    d.N_max = 65
    assert lib.specvlm_tree_verify_attn_workspace_bytes(ctypes.byref(d)) == 0
    d.N_max = 60
    null = ctypes.c_void_p(None)
    rc = lib.specvlm_tree_verify_attn(ctypes.byref(d), null, null, null, null, null, null, null, null, null,
                                      null, 0, null, null)
    assert rc == 1                                                                      # INVALID_ARG
    assert lib.specvlm_node_argmax(0, 1, 65, 10, null, 0, 10, null, null, null) == 1
    assert lib.specvlm_tree_accept(1, 8, 0, *([null] * 10)) == 1
    # draft-side growth: K > V, K > 64, too many candidates, N_max > 64
    assert lib.specvlm_draft_topk(0, 1, 1, 10, 11, *([null, 0, 10] + [null, 0] * 2 + [null] * 3 + [11, null, null])) == 1
    assert lib.specvlm_draft_topk(0, 1, 1, 100, 65, *([null, 0, 100] + [null, 0] * 2 + [null] * 3 + [65, null, null])) == 1
    assert lib.specvlm_draft_select(1, 8193, 4, null, 8193, null, 0, null, null, null, null) == 1
    # fused level: more than 1024 new candidates, or no ticket counters (pointers are never touched: the checks come first)
    fake = ctypes.c_void_p(4096)
    level = [fake, 0, 32000, null, 0, null, 0, fake, fake, null]
    assert lib.specvlm_draft_topk_select(0, 1, 103, 32000, 10, *level, 1030, null, 10, 0, fake, null, null, fake, null) == 1
    assert lib.specvlm_draft_topk_select(0, 1, 10, 32000, 10, *level, 100, null, 10, 0, fake, null, null, null, null) == 1
    assert lib.specvlm_draft_topk_select(0, 1, 10, 32000, 10, *level, 100, null, 0, 0, fake, null, null, fake, null) == 1
    assert lib.specvlm_draft_finalize(1, 100, 65, null, null, null, 100, *([null] * 8)) == 1


def test_split_choice_and_workspace_sizes_for_the_five_workloads():
    """Host logic only: the library's key-range split count and workspace size for the shapes of the
    five workload configurations (one workgroup per compute unit where the batch allows it)."""
    import paper_2509_11815_amd as sv
    from paper_2509_11815_amd.binding import AttnDesc
    lib = sv.load_library()

    def desc(B, H, D, N, cap, paged=False, dtype=0):
        d = AttnDesc()
        d.dtype, d.B, d.H_q, d.H_kv, d.D, d.N_max = dtype, B, H, H, D, N
        d.q_stride_b, d.q_stride_n, d.q_stride_h = N * H * D, H * D, D
        d.o_stride_b, d.o_stride_n, d.o_stride_h = N * H * D, H * D, D
        if paged:
            d.paged, d.block_size, d.max_blocks_per_req, d.num_blocks = 1, 16, cap // 16, B * cap // 16 + 8
            d.kv_stride_b, d.kv_stride_h, d.kv_stride_t = H * 16 * D, 16 * D, D
        else:
            d.kv_capacity = cap
            d.kv_stride_b, d.kv_stride_h, d.kv_stride_t = H * cap * D, cap * D, D
        return d

    cases = {"C1": (desc(1, 4, 64, 8, 80, dtype=1), 1), "C2": (desc(1, 32, 128, 60, 832), 7),
             "C3": (desc(1, 32, 128, 60, 3328), 8), "C4": (desc(8, 32, 128, 60, 976), 1),
             "C5": (desc(4, 40, 128, 60, 4928, paged=True), 3)}
    for name, (d, want) in cases.items():
        got = lib.specvlm_tree_verify_attn_num_splits(ctypes.byref(d))
        assert got == want, (name, got)
        need = lib.specvlm_tree_verify_attn_workspace_bytes(ctypes.byref(d))
        if d.dtype == 0 and want > 1:
            parts = d.B * d.H_q * want
            counters = 1024 * 4 * 128                                            # a fixed region, whatever the shape: a 128-byte line per counter
            assert need == counters + parts * (64 * d.D * 2 + 64 * 8), name     # bf16 partials + (max, sum) pairs
    d = cases["C3"][0]
    d.num_splits = 5                                                             # a caller's choice is kept
    assert lib.specvlm_tree_verify_attn_num_splits(ctypes.byref(d)) == 5
    d.num_splits = 64                                                            # ... up to SPECVLM_MAX_SPLITS
    assert lib.specvlm_tree_verify_attn_num_splits(ctypes.byref(d)) == 64
    for bad in (65, 1000, -1):                                                   # outside the documented range 0 .. 64
        d.num_splits = bad
        assert lib.specvlm_tree_verify_attn_num_splits(ctypes.byref(d)) == 0
        assert lib.specvlm_tree_verify_attn_workspace_bytes(ctypes.byref(d)) == 0
    d.num_splits, d.B, d.H_q, d.H_kv = 8, 9, 128, 128                            # 1152 (request, head) pairs: unsplit
    assert lib.specvlm_tree_verify_attn_num_splits(ctypes.byref(d)) == 1
    d.num_splits, d.B, d.H_q, d.H_kv = 0, 1, 32, 32
    assert lib.specvlm_head_argmax_workspace_bytes(1, 60, 32000) == 256 + 250 * 64 * 8
    assert lib.specvlm_head_argmax_workspace_bytes(8, 60, 32000) == 256 + 8 * 250 * 64 * 8
    assert lib.specvlm_head_argmax_workspace_bytes(0, 60, 32000) == 0


def test_attention_kernels_spill_nothing():
    """The matrix-core attention kernels count their outstanding memory operations by hand
    (s_waitcnt vmcnt) and read results of hand-written loads after hand-written waits: a register
    spilled to scratch memory would add memory operations the count does not know, and could save a
    register before its load has landed.  So they must compile without scratch, and the shape
    meant for two workgroups per compute unit must stay within 128 registers and half the LDS."""
    from paper_2509_11815_amd import build
    usage = build.kernel_resource_usage("attn_mfma.hip")
    kernels = {k: v for k, v in usage.items() if "attn_mfma_kernel" in k}
    assert len(kernels) == 4, sorted(usage)                    # two shapes x two head sizes
    for name, u in kernels.items():
        assert u["scratch"] == 0, (name, u)
        if "2wg" in name:
            assert u["vgprs"] <= 128 and u["lds"] <= 80 * 1024, (name, u)
        else:
            assert u["lds"] <= 160 * 1024, (name, u)


def test_binding_constants_are_the_headers():
    import re
    from paper_2509_11815_amd import binding
    text = open(os.path.join(ROOT, "include", "specvlm.h")).read()
    assert int(re.search(r"#define SPECVLM_COUNTER_STRIDE (\d+)", text).group(1)) == binding.COUNTER_STRIDE
