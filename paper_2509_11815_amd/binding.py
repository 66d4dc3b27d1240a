"""ctypes binding of libspecvlm.so: same names as the C entry points, marshalling only.

Every step runs in the library's HIP kernels; there is no fallback.  Importing this module
does not need the library; the first call loads it and raises if it has not been built
(``python -m paper_2509_11815_amd.build``).
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

SPECVLM_BF16, SPECVLM_F32 = 0, 1
STATUS = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "WORKSPACE_TOO_SMALL", 4: "HIP_ERROR"}
ERR_BITS = {1: "BAD_PARENT", 2: "BAD_NUM_NODES", 4: "BAD_LENGTH", 8: "PATH_TOO_LONG", 16: "BAD_BLOCK",
            32: "BAD_TOKEN", 64: "TREE_NOT_CLOSED"}


def err_flag_names(word: int) -> list[str]:
    """Names of the SPECVLM_ERR_* bits set in a device error word (after the caller synchronised)."""
    return [name for bit, name in ERR_BITS.items() if word & bit] + (
        [hex(word & ~sum(ERR_BITS))] if word & ~sum(ERR_BITS) else [])

EXPORTS = ["specvlm_version", "specvlm_last_hip_error", "specvlm_tree_verify_attn_workspace_bytes",
           "specvlm_tree_verify_attn_num_splits",
           "specvlm_tree_verify_attn", "specvlm_tree_verify_attn_static", "specvlm_tree_verify_attn_vector_alu",
           "specvlm_node_argmax", "specvlm_tree_accept", "specvlm_tree_accept_sample",
           "specvlm_kv_compact", "specvlm_draft_topk", "specvlm_draft_topk_select", "specvlm_draft_select",
           "specvlm_draft_finalize",
           "specvlm_head_argmax", "specvlm_head_argmax_workspace_bytes",
           "specvlm_visual_pool", "specvlm_visual_prune", "specvlm_node_argmax_accept"]


class SpecvlmError(RuntimeError):
    pass


class AttnDesc(ctypes.Structure):
    """Mirror of specvlm_attn_desc."""
    _fields_ = [("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("H_q", ctypes.c_int32),
                ("H_kv", ctypes.c_int32), ("D", ctypes.c_int32), ("N_max", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("paged", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("max_blocks_per_req", ctypes.c_int32),
                ("num_blocks", ctypes.c_int32), ("kv_capacity", ctypes.c_int32),
                ("num_splits", ctypes.c_int32),
                ("q_stride_b", ctypes.c_int64), ("q_stride_n", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
                ("o_stride_b", ctypes.c_int64), ("o_stride_n", ctypes.c_int64), ("o_stride_h", ctypes.c_int64),
                ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64), ("kv_stride_t", ctypes.c_int64)]


_lib = None


def load_library(path: str | None = None) -> ctypes.CDLL:
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("SPECVLM_LIB") or _build.LIB       # SPECVLM_LIB: alternative build of the library
    if not os.path.exists(path):
        raise SpecvlmError(f"{path} is missing: build it with `python -m paper_2509_11815_amd.build` "
                           "(there is no fallback path)")
    L = ctypes.CDLL(path)
    missing = [name for name in EXPORTS if not hasattr(L, name)]
    if missing:
        raise SpecvlmError(f"{path} does not export {missing}: rebuild it with `python -m paper_2509_11815_amd.build`")
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.specvlm_version.restype = i32
    L.specvlm_last_hip_error.restype = i32
    L.specvlm_tree_verify_attn_workspace_bytes.restype = ctypes.c_size_t
    L.specvlm_tree_verify_attn_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
    L.specvlm_tree_verify_attn_num_splits.restype = i32
    L.specvlm_tree_verify_attn_num_splits.argtypes = [ctypes.POINTER(AttnDesc)]
    L.specvlm_tree_verify_attn.restype = i32
    L.specvlm_tree_verify_attn.argtypes = [ctypes.POINTER(AttnDesc)] + [vp] * 9 + [vp, ctypes.c_size_t, vp, vp]
    L.specvlm_tree_verify_attn_static.restype = i32
    L.specvlm_tree_verify_attn_static.argtypes = [ctypes.POINTER(AttnDesc)] + [vp] * 9 + [vp, vp]
    L.specvlm_node_argmax.restype = i32
    L.specvlm_node_argmax.argtypes = [i32, i32, i32, i32, vp, i64, i64, vp, vp, vp]
    L.specvlm_tree_accept.restype = i32
    L.specvlm_tree_accept.argtypes = [i32, i32, i32] + [vp] * 10
    L.specvlm_tree_accept_sample.restype = i32
    L.specvlm_tree_accept_sample.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, i64, i64, vp, ctypes.c_float] + [vp] * 8
    L.specvlm_kv_compact.restype = i32
    L.specvlm_kv_compact.argtypes = [ctypes.POINTER(AttnDesc), i32, vp, vp, i64, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
    L.specvlm_tree_verify_attn_vector_alu.restype = i32
    L.specvlm_tree_verify_attn_vector_alu.argtypes = [ctypes.POINTER(AttnDesc)] + [vp] * 9 + [vp, vp]
    L.specvlm_draft_topk.restype = i32
    L.specvlm_draft_topk.argtypes = [i32] * 5 + [vp, i64, i64, vp, i64, vp, i64, vp, vp, vp, i64, vp, vp]
    L.specvlm_draft_topk_select.restype = i32
    L.specvlm_draft_topk_select.argtypes = ([i32] * 5 + [vp, i64, i64, vp, i64, vp, i64, vp, vp, vp, i64, vp] +
                                            [i32, i32, vp, vp, vp, vp, vp])
    L.specvlm_draft_select.restype = i32
    L.specvlm_draft_select.argtypes = [i32, i32, i32, vp, i64, vp, i32, vp, vp, vp, vp]
    L.specvlm_draft_finalize.restype = i32
    L.specvlm_draft_finalize.argtypes = [i32, i32, i32, vp, vp, vp, i64] + [vp] * 8
    L.specvlm_head_argmax_workspace_bytes.restype = ctypes.c_size_t
    L.specvlm_head_argmax_workspace_bytes.argtypes = [i32, i32, i32]
    L.specvlm_head_argmax.restype = i32
    L.specvlm_head_argmax.argtypes = [i32] * 5 + [vp, i64, i64, vp, i64, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.specvlm_visual_pool.restype = i32
    L.specvlm_visual_pool.argtypes = [i32] * 5 + [vp, i64, i64, vp, vp, i64, i64, vp, vp, vp]
    L.specvlm_visual_prune.restype = i32
    L.specvlm_visual_prune.argtypes = [i32] * 5 + [vp, i64, i64, vp, vp, i64, i64, vp, vp]
    L.specvlm_node_argmax_accept.restype = i32
    L.specvlm_node_argmax_accept.argtypes = [i32] * 5 + [vp, i64, i64] + [vp] * 11
    _lib = L
    return L


def lib() -> ctypes.CDLL:
    return load_library()


def _check(rc: int, what: str):
    if rc != 0:
        extra = f" (hipError {lib().specvlm_last_hip_error()})" if rc == 4 else ""
        raise SpecvlmError(f"{what}: {STATUS.get(rc, rc)}{extra}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return SPECVLM_BF16
    if t.dtype == torch.float32:
        return SPECVLM_F32
    raise TypeError(f"bfloat16 or float32 expected, got {t.dtype}")


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev_i32(t, name):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous int32 device tensor")
    return t


COUNTER_STRIDE = 32                 # SPECVLM_COUNTER_STRIDE: int32 words between two requests' arrival counters


def _request_counters(counters, B, dev):
    """The per-request arrival counters of the fused calls: allocated (zeroed) when omitted, else checked."""
    if counters is None:
        return torch.zeros(B * COUNTER_STRIDE, dtype=torch.int32, device=dev)
    _dev_i32(counters, "counters")
    if counters.numel() < B * COUNTER_STRIDE:
        raise ValueError(f"counters must hold B * COUNTER_STRIDE = {B * COUNTER_STRIDE} int32 words")
    return counters


def make_attn_desc(q, k_cache, out=None, *, block_table=None, softmax_scale=0.0, num_splits=0) -> AttnDesc:
    """Fill a specvlm_attn_desc from tensor shapes and strides.

    q [B,N_max,H_q,D]; contiguous cache [B,H_kv,capacity,D]; paged cache [num_blocks,H_kv,16,D]."""
    B, N_max, H_q, D = q.shape
    d = AttnDesc()
    d.dtype = _dtype_code(q)
    d.B, d.H_q, d.H_kv, d.D, d.N_max = B, H_q, k_cache.shape[1], D, N_max
    d.softmax_scale = float(softmax_scale)
    d.num_splits = int(num_splits)
    if q.stride(3) != 1 or k_cache.stride(3) != 1:
        raise ValueError("innermost dimension must be contiguous")
    d.q_stride_b, d.q_stride_n, d.q_stride_h = q.stride(0), q.stride(1), q.stride(2)
    o = q if out is None else out
    d.o_stride_b, d.o_stride_n, d.o_stride_h = o.stride(0), o.stride(1), o.stride(2)
    d.kv_stride_b, d.kv_stride_h, d.kv_stride_t = k_cache.stride(0), k_cache.stride(1), k_cache.stride(2)
    if block_table is not None:
        d.paged, d.block_size = 1, k_cache.shape[2]
        d.max_blocks_per_req = block_table.shape[1]
        d.num_blocks = k_cache.shape[0]
        d.kv_capacity = d.max_blocks_per_req * d.block_size
    else:
        d.paged, d.block_size, d.max_blocks_per_req, d.num_blocks = 0, 0, 0, 0
        d.kv_capacity = k_cache.shape[2]
    return d


def specvlm_version() -> int:
    return int(lib().specvlm_version())


def specvlm_tree_verify_attn_workspace_bytes(desc: AttnDesc) -> int:
    return int(lib().specvlm_tree_verify_attn_workspace_bytes(ctypes.byref(desc)))


def specvlm_tree_verify_attn_num_splits(desc: AttnDesc) -> int:
    return int(lib().specvlm_tree_verify_attn_num_splits(ctypes.byref(desc)))


def specvlm_tree_verify_attn(q, k_cache, v_cache, prefix_len, parent, *, num_nodes=None, block_table=None,
                             out=None, lse=None, workspace=None, err_flag=None, softmax_scale=0.0,
                             num_splits=0, desc=None, stream=None):
    """One layer of tree-masked verification attention.  Returns `out` ([B,N_max,H_q,D])."""
    if out is None:
        out = torch.zeros_like(q)
    if desc is None:
        desc = make_attn_desc(q, k_cache, out, block_table=block_table, softmax_scale=softmax_scale,
                              num_splits=num_splits)
    if k_cache.stride() != v_cache.stride() or k_cache.shape != v_cache.shape:
        raise ValueError("K and V caches must share one geometry")
    need = specvlm_tree_verify_attn_workspace_bytes(desc)
    if workspace is None and need:
        workspace = torch.zeros(need, dtype=torch.uint8, device=q.device)   # zero-filled once, as the ABI asks
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().specvlm_tree_verify_attn(
        ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(_dev_i32(block_table, "block_table")),
        _ptr(_dev_i32(prefix_len, "prefix_len")), _ptr(_dev_i32(num_nodes, "num_nodes")),
        _ptr(_dev_i32(parent, "parent")), _ptr(out), _ptr(lse), _ptr(workspace), ctypes.c_size_t(wbytes),
        _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_tree_verify_attn")
    return out


def specvlm_tree_verify_attn_vector_alu(q, k_cache, v_cache, prefix_len, parent, *, out, **kw):
    """Measurement aid: the same call computed by the vector-ALU kernel (see the header)."""
    return specvlm_tree_verify_attn_static(q, k_cache, v_cache, prefix_len, parent, out=out,
                                           _entry="specvlm_tree_verify_attn_vector_alu", **kw)


def specvlm_tree_verify_attn_static(q, k_cache, v_cache, prefix_len, parent, *, out, num_nodes=None,
                                    block_table=None, lse=None, err_flag=None, softmax_scale=0.0,
                                    num_splits=0, desc=None, stream=None, _entry="specvlm_tree_verify_attn_static"):
    """specvlm_tree_verify_attn on the library's own static scratch array.  Allocates nothing: `out`
    (and `lse`) must be supplied."""
    if desc is None:
        desc = make_attn_desc(q, k_cache, out, block_table=block_table, softmax_scale=softmax_scale,
                              num_splits=num_splits)
    if k_cache.stride() != v_cache.stride() or k_cache.shape != v_cache.shape:
        raise ValueError("K and V caches must share one geometry")
    rc = getattr(lib(), _entry)(
        ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(_dev_i32(block_table, "block_table")),
        _ptr(_dev_i32(prefix_len, "prefix_len")), _ptr(_dev_i32(num_nodes, "num_nodes")),
        _ptr(_dev_i32(parent, "parent")), _ptr(out), _ptr(lse), _ptr(err_flag), _stream(stream))
    _check(rc, _entry)
    return out


def specvlm_node_argmax(logits, *, num_nodes=None, out=None, stream=None):
    """logits [B,N_max,V] -> int32 [B,N_max] lowest index of each row's maximum."""
    B, N_max, V = logits.shape
    if logits.stride(2) != 1:
        raise ValueError("vocab dimension must be contiguous")
    if out is None:
        out = torch.empty((B, N_max), dtype=torch.int32, device=logits.device)
    rc = lib().specvlm_node_argmax(_dtype_code(logits), B, N_max, V, _ptr(logits), logits.stride(0),
                                   logits.stride(1), _ptr(_dev_i32(num_nodes, "num_nodes")), _ptr(out),
                                   _stream(stream))
    _check(rc, "specvlm_node_argmax")
    return out


def specvlm_tree_accept(parent, draft_tok, amax, *, num_nodes=None, path_cap=8, err_flag=None, out=None,
                        stream=None):
    """Returns (accept_len [B], path [B,path_cap], bonus_tok [B], committed_tok [B,path_cap]);
    `out` may supply these four int32 device tensors."""
    B, N_max = parent.shape
    dev = parent.device
    if out is not None:
        accept_len, path, bonus, committed = out
        path_cap = path.shape[1]
    else:
        accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        path = torch.empty((B, path_cap), dtype=torch.int32, device=dev)
        bonus = torch.empty(B, dtype=torch.int32, device=dev)
        committed = torch.empty((B, path_cap), dtype=torch.int32, device=dev)
    rc = lib().specvlm_tree_accept(B, N_max, path_cap, _ptr(_dev_i32(parent, "parent")),
                                   _ptr(_dev_i32(draft_tok, "draft_tok")), _ptr(_dev_i32(amax, "amax")),
                                   _ptr(_dev_i32(num_nodes, "num_nodes")), _ptr(accept_len), _ptr(path),
                                   _ptr(bonus), _ptr(committed), _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_tree_accept")
    return accept_len, path, bonus, committed


def specvlm_tree_accept_sample(parent, draft_tok, logits, u_accept, u_bonus, *, temperature=1.0, num_nodes=None,
                               path_cap=8, err_flag=None, out=None, stream=None):
    """Sampling-based acceptance (temperature > 0).  logits [B,N_max,V]; u_accept [B,N_max] and u_bonus [B]
    fp32 uniform numbers in [0,1).  Returns (accept_len, path, bonus_tok, committed_tok) like
    specvlm_tree_accept."""
    B, N_max, V = logits.shape
    dev = logits.device
    if logits.stride(2) != 1:
        raise ValueError("vocab dimension must be contiguous")
    for name, t, shape in (("u_accept", u_accept, (B, N_max)), ("u_bonus", u_bonus, (B,))):
        if t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous float32 tensor of shape {shape}")
    if out is not None:
        accept_len, path, bonus, committed = out
        path_cap = path.shape[1]
    else:
        accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        path = torch.empty((B, path_cap), dtype=torch.int32, device=dev)
        bonus = torch.empty(B, dtype=torch.int32, device=dev)
        committed = torch.empty((B, path_cap), dtype=torch.int32, device=dev)
    rc = lib().specvlm_tree_accept_sample(
        _dtype_code(logits), B, N_max, V, path_cap, _ptr(_dev_i32(parent, "parent")),
        _ptr(_dev_i32(draft_tok, "draft_tok")), _ptr(logits), logits.stride(0), logits.stride(1),
        _ptr(_dev_i32(num_nodes, "num_nodes")), ctypes.c_float(temperature), _ptr(u_accept), _ptr(u_bonus),
        _ptr(accept_len), _ptr(path), _ptr(bonus), _ptr(committed), _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_tree_accept_sample")
    return accept_len, path, bonus, committed


def specvlm_kv_compact(k_caches, v_caches, prefix_len, path, accept_len, *, block_table=None,
                       new_prefix_len=None, moved_idx=None, layer_ptrs=None, err_flag=None, stream=None):
    """In-place compaction.  k_caches/v_caches: one tensor [L, <per-layer cache dims>] (layer stride taken
    from the tensor), or with `layer_ptrs=(k_ptrs, v_ptrs)` (int64 device tensors of L addresses) a single
    layer's tensor that only provides the geometry.  Returns (new_prefix_len, moved_idx)."""
    B, path_cap = path.shape
    dev = path.device
    if new_prefix_len is None:
        new_prefix_len = torch.empty(B, dtype=torch.int32, device=dev)
    if layer_ptrs is None:
        L = k_caches.shape[0]
        layer0 = k_caches[0]
        layer_stride = k_caches.stride(0)
        kb, vb, kp, vp = _ptr(k_caches), _ptr(v_caches), None, None
        if k_caches.stride() != v_caches.stride():
            raise ValueError("K and V caches must share one geometry")
    else:
        kp_t, vp_t = layer_ptrs
        L = kp_t.numel()
        layer0 = k_caches
        layer_stride = 0
        kb, vb, kp, vp = None, None, _ptr(kp_t), _ptr(vp_t)
    d = AttnDesc()
    d.dtype = _dtype_code(layer0)
    d.B, d.H_q, d.H_kv, d.D, d.N_max = B, layer0.shape[1], layer0.shape[1], layer0.shape[3], 64
    d.kv_stride_b, d.kv_stride_h, d.kv_stride_t = layer0.stride(0), layer0.stride(1), layer0.stride(2)
    if block_table is not None:
        d.paged, d.block_size = 1, layer0.shape[2]
        d.max_blocks_per_req = block_table.shape[1]
        d.num_blocks = layer0.shape[0]
        d.kv_capacity = d.max_blocks_per_req * d.block_size
    else:
        d.kv_capacity = layer0.shape[2]
    rc = lib().specvlm_kv_compact(ctypes.byref(d), L, kb, vb, layer_stride, kp, vp,
                                  _ptr(_dev_i32(block_table, "block_table")),
                                  _ptr(_dev_i32(prefix_len, "prefix_len")), _ptr(_dev_i32(path, "path")),
                                  path_cap, _ptr(_dev_i32(accept_len, "accept_len")), _ptr(new_prefix_len),
                                  _ptr(moved_idx), _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_kv_compact")
    return new_prefix_len, moved_idx


def _dev_f32(t, name):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.float32 and t.stride(-1) == 1):
        raise TypeError(f"{name} must be a float32 device tensor with a contiguous last dimension")
    return t


def specvlm_draft_topk(logits, K, *, cum=None, parent_idx=None, score_out=None, token_out=None, parent_out=None,
                       lse_out=None, stream=None):
    """One level of draft-tree growth.  logits [B,W,V]; cum fp32 / parent_idx int32 [B,W] (row strides are
    taken from the tensors, so they may be views).  Outputs are [B, >= W*K] fp32 / int32 tensors or views
    (row stride taken from score_out; token_out and parent_out must share it): entry (b, w*K + k).
    Returns (score_out, token_out, parent_out)."""
    B, W, V = logits.shape
    dev = logits.device
    if logits.stride(2) != 1:
        raise ValueError("vocab dimension must be contiguous")
    if score_out is None:
        score_out = torch.empty((B, W * K), dtype=torch.float32, device=dev)
    if token_out is None:
        token_out = torch.empty((B, W * K), dtype=torch.int32, device=dev)
    if parent_out is None and parent_idx is not None:
        parent_out = torch.empty((B, W * K), dtype=torch.int32, device=dev)
    outs = [t for t in (score_out, token_out, parent_out) if t is not None]
    if any(t.stride(0) != score_out.stride(0) or t.stride(1) != 1 or t.shape[1] < W * K for t in outs):
        raise ValueError("score_out / token_out / parent_out must share one row stride and hold W*K entries")
    if token_out.dtype != torch.int32 or (parent_out is not None and parent_out.dtype != torch.int32):
        raise TypeError("token_out / parent_out must be int32")
    _dev_f32(score_out, "score_out")
    rc = lib().specvlm_draft_topk(
        _dtype_code(logits), B, W, V, K, _ptr(logits), logits.stride(0), logits.stride(1),
        _ptr(_dev_f32(cum, "cum")), 0 if cum is None else cum.stride(0),
        _ptr(parent_idx), 0 if parent_idx is None else parent_idx.stride(0),
        _ptr(score_out), _ptr(token_out), _ptr(parent_out), score_out.stride(0), _ptr(_dev_f32(lse_out, "lse_out")),
        _stream(stream))
    _check(rc, "specvlm_draft_topk")
    return score_out, token_out, parent_out


def specvlm_draft_topk_select(logits, K, M, *, cum=None, parent_idx=None, score_out=None, token_out=None,
                              parent_out=None, lse_out=None, index_base=0, sel_out=None, sel_score_out=None,
                              count_out=None, counters=None, stream=None):
    """specvlm_draft_topk and the selection of the M best of the level's W*K new candidates in one launch.
    `counters` is an int32 [B * COUNTER_STRIDE] device tensor, zero-filled once (allocated here when
    omitted).  Returns (score_out, token_out, parent_out, sel_out, sel_score_out, count_out)."""
    B, W, V = logits.shape
    dev = logits.device
    if logits.stride(2) != 1:
        raise ValueError("vocab dimension must be contiguous")
    if score_out is None:
        score_out = torch.empty((B, W * K), dtype=torch.float32, device=dev)
    if token_out is None:
        token_out = torch.empty((B, W * K), dtype=torch.int32, device=dev)
    if parent_out is None and parent_idx is not None:
        parent_out = torch.empty((B, W * K), dtype=torch.int32, device=dev)
    outs = [t for t in (score_out, token_out, parent_out) if t is not None]
    if any(t.stride(0) != score_out.stride(0) or t.stride(1) != 1 or t.shape[1] < W * K for t in outs):
        raise ValueError("score_out / token_out / parent_out must share one row stride and hold W*K entries")
    if token_out.dtype != torch.int32 or (parent_out is not None and parent_out.dtype != torch.int32):
        raise TypeError("token_out / parent_out must be int32")
    _dev_f32(score_out, "score_out")
    if sel_out is None:
        sel_out = torch.empty((B, M), dtype=torch.int32, device=dev)
    if sel_score_out is None:
        sel_score_out = torch.empty((B, M), dtype=torch.float32, device=dev)
    if count_out is None:
        count_out = torch.empty(B, dtype=torch.int32, device=dev)
    counters = _request_counters(counters, B, dev)
    rc = lib().specvlm_draft_topk_select(
        _dtype_code(logits), B, W, V, K, _ptr(logits), logits.stride(0), logits.stride(1),
        _ptr(_dev_f32(cum, "cum")), 0 if cum is None else cum.stride(0),
        _ptr(parent_idx), 0 if parent_idx is None else parent_idx.stride(0),
        _ptr(score_out), _ptr(token_out), _ptr(parent_out), score_out.stride(0), _ptr(_dev_f32(lse_out, "lse_out")),
        M, index_base, _ptr(_dev_i32(sel_out, "sel_out")), _ptr(_dev_f32(sel_score_out, "sel_score_out")),
        _ptr(_dev_i32(count_out, "count_out")), _ptr(_dev_i32(counters, "counters")), _stream(stream))
    _check(rc, "specvlm_draft_topk_select")
    return score_out, token_out, parent_out, sel_out, sel_score_out, count_out


def specvlm_draft_select(score, M, *, num_cand=None, index_base=0, sel_out=None, sel_score_out=None,
                         count_out=None, stream=None):
    """score fp32 [B,C] (may be a view of a wider array).  Returns (sel [B,M] int32, sel_score [B,M] fp32,
    count [B] int32)."""
    B, C = score.shape
    dev = score.device
    _dev_f32(score, "score")
    if sel_out is None:
        sel_out = torch.empty((B, M), dtype=torch.int32, device=dev)
    if sel_score_out is None:
        sel_score_out = torch.empty((B, M), dtype=torch.float32, device=dev)
    if count_out is None:
        count_out = torch.empty(B, dtype=torch.int32, device=dev)
    rc = lib().specvlm_draft_select(B, C, M, _ptr(score), score.stride(0), _ptr(_dev_i32(num_cand, "num_cand")),
                                    index_base, _ptr(_dev_i32(sel_out, "sel_out")), _ptr(sel_score_out),
                                    _ptr(_dev_i32(count_out, "count_out")), _stream(stream))
    _check(rc, "specvlm_draft_select")
    return sel_out, sel_score_out, count_out


def specvlm_draft_finalize(cand_score, cand_parent, cand_token, root_token, N_max, *, num_cand=None, err_flag=None,
                           out=None, stream=None):
    """Candidates [B,C] (fp32 score, int32 parent and token, one row stride) -> (parent [B,N_max],
    draft_tok [B,N_max], node_cand [B,N_max], num_nodes [B]); `out` may supply these four int32 tensors."""
    B, C = cand_score.shape
    dev = cand_score.device
    _dev_f32(cand_score, "cand_score")
    for t in (cand_parent, cand_token):
        if t.dtype != torch.int32 or t.stride() != cand_score.stride():
            raise ValueError("cand_parent / cand_token must be int32 with cand_score's strides")
    if out is not None:
        parent, tok, node_cand, num_nodes = out
    else:
        parent = torch.empty((B, N_max), dtype=torch.int32, device=dev)
        tok = torch.empty((B, N_max), dtype=torch.int32, device=dev)
        node_cand = torch.empty((B, N_max), dtype=torch.int32, device=dev)
        num_nodes = torch.empty(B, dtype=torch.int32, device=dev)
    rc = lib().specvlm_draft_finalize(
        B, C, N_max, _ptr(cand_score), _ptr(cand_parent), _ptr(cand_token), cand_score.stride(0),
        _ptr(_dev_i32(num_cand, "num_cand")), _ptr(_dev_i32(root_token, "root_token")),
        _ptr(_dev_i32(parent, "parent")), _ptr(_dev_i32(tok, "draft_tok")), _ptr(node_cand),
        _ptr(_dev_i32(num_nodes, "num_nodes")), _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_draft_finalize")
    return parent, tok, node_cand, num_nodes


def specvlm_head_argmax_workspace_bytes(B, N_max, V) -> int:
    return int(lib().specvlm_head_argmax_workspace_bytes(B, N_max, V))


def specvlm_head_argmax(hidden, weight, *, num_nodes=None, out=None, max_logit=None, workspace=None, stream=None):
    """Output head fused with the greedy choice.  hidden [B,N_max,E] bf16, weight [V,E] bf16 ->
    amax [B,N_max] int32 (and the greatest logit into `max_logit` fp32 [B,N_max] if given)."""
    B, N_max, E = hidden.shape
    V = weight.shape[0]
    if hidden.stride(2) != 1 or weight.stride(1) != 1 or weight.shape[1] != E:
        raise ValueError("hidden [B,N_max,E] and weight [V,E] need a contiguous last dimension of equal size")
    if out is None:
        out = torch.empty((B, N_max), dtype=torch.int32, device=hidden.device)
    need = specvlm_head_argmax_workspace_bytes(B, N_max, V)
    if workspace is None:
        workspace = torch.zeros(need, dtype=torch.uint8, device=hidden.device)   # zero-filled once, as the ABI asks
    rc = lib().specvlm_head_argmax(
        _dtype_code(hidden), B, N_max, E, V, _ptr(hidden), hidden.stride(0), hidden.stride(1), _ptr(weight),
        weight.stride(0), _ptr(_dev_i32(num_nodes, "num_nodes")), _ptr(_dev_i32(out, "out")),
        _ptr(_dev_f32(max_logit, "max_logit")), _ptr(workspace),
        ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    _check(rc, "specvlm_head_argmax")
    return out


def specvlm_visual_pool(x, ratio, *, num_tokens=None, out=None, out_tokens=None, err_flag=None, stream=None):
    """Average pooling along the token sequence (window = stride = ratio, ragged last window).
    x [B,T,E] -> (y [B,ceil(T/ratio),E], out_tokens [B] int32)."""
    B, T, E = x.shape
    Tp = (T + ratio - 1) // ratio if ratio > 0 else T      # (the library rejects ratio < 1)
    if out is None:
        out = torch.zeros((B, Tp, E), dtype=x.dtype, device=x.device)
    if out_tokens is None:
        out_tokens = torch.empty(B, dtype=torch.int32, device=x.device)
    if x.stride(2) != 1 or out.stride(2) != 1:
        raise ValueError("feature dimension must be contiguous")
    rc = lib().specvlm_visual_pool(_dtype_code(x), B, T, E, ratio, _ptr(x), x.stride(0), x.stride(1),
                                   _ptr(_dev_i32(num_tokens, "num_tokens")), _ptr(out), out.stride(0), out.stride(1),
                                   _ptr(_dev_i32(out_tokens, "out_tokens")), _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_visual_pool")
    return out, out_tokens


def specvlm_visual_prune(x, keep, *, out=None, err_flag=None, stream=None):
    """Pruning as a gather: x [B,T,E], keep [B,T_keep] int32 (-1 = padding) -> y [B,T_keep,E]."""
    B, T, E = x.shape
    T_keep = keep.shape[1]
    if out is None:
        out = torch.zeros((B, T_keep, E), dtype=x.dtype, device=x.device)
    if x.stride(2) != 1 or out.stride(2) != 1:
        raise ValueError("feature dimension must be contiguous")
    rc = lib().specvlm_visual_prune(_dtype_code(x), B, T, T_keep, E, _ptr(x), x.stride(0), x.stride(1),
                                    _ptr(_dev_i32(keep, "keep")), _ptr(out), out.stride(0), out.stride(1),
                                    _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_visual_prune")
    return out


def specvlm_node_argmax_accept(logits, parent, draft_tok, *, num_nodes=None, path_cap=8, counters=None, amax=None,
                               err_flag=None, out=None, stream=None):
    """specvlm_node_argmax + specvlm_tree_accept in one launch.  `counters` is an int32
    [B * COUNTER_STRIDE] device tensor, zero-filled once (allocated here when omitted).
    Returns (amax, accept_len, path, bonus_tok, committed_tok)."""
    B, N_max, V = logits.shape
    dev = logits.device
    if logits.stride(2) != 1:
        raise ValueError("vocab dimension must be contiguous")
    if out is not None:
        accept_len, path, bonus, committed = out
        path_cap = path.shape[1]
    else:
        accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        path = torch.empty((B, path_cap), dtype=torch.int32, device=dev)
        bonus = torch.empty(B, dtype=torch.int32, device=dev)
        committed = torch.empty((B, path_cap), dtype=torch.int32, device=dev)
    if amax is None:
        amax = torch.empty((B, N_max), dtype=torch.int32, device=dev)
    counters = _request_counters(counters, B, dev)
    rc = lib().specvlm_node_argmax_accept(
        _dtype_code(logits), B, N_max, V, path_cap, _ptr(logits), logits.stride(0), logits.stride(1),
        _ptr(_dev_i32(num_nodes, "num_nodes")), _ptr(_dev_i32(parent, "parent")),
        _ptr(_dev_i32(draft_tok, "draft_tok")), _ptr(_dev_i32(amax, "amax")), _ptr(accept_len), _ptr(path),
        _ptr(bonus), _ptr(committed), _ptr(_dev_i32(counters, "counters")), _ptr(err_flag), _stream(stream))
    _check(rc, "specvlm_node_argmax_accept")
    return amax, accept_len, path, bonus, committed
