"""fp64 CPU oracle for the tree-verification step -- TEST INFRASTRUCTURE.

Thin ctypes/numpy front end of ``specvlm_oracle.c`` (same directory), which
holds the plain definitions (SpecVLM Sec. 3.1 verification, Sec. 4.1 tree
attention).  Only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does.
It shares no code with the HIP library.

bf16 tensors are passed as ``uint16`` bit patterns, fp32 as ``float32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "specvlm_oracle.c")
_LIB = os.path.join(_HERE, "libspecvlm_oracle.so")
_lib = None

BF16, F32 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over heads/nodes only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float32:
        return F32
    raise TypeError(f"oracle takes uint16 (bf16 bits) or float32, got {a.dtype}")


def _estrides(a: np.ndarray):
    return [s // a.itemsize for s in a.strides]


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def ancestors(parent):
    """(anc [n,n] uint8, depth [n] int32) of one parent array."""
    parent = _i32(parent)
    n = parent.shape[0]
    anc = np.zeros((n, n), dtype=np.uint8)
    depth = np.zeros(n, dtype=np.int32)
    rc = _load().oracle_ancestors(ctypes.c_int(n), _p(parent), _p(anc), _p(depth))
    if rc:
        raise ValueError("parent array is not a topologically ordered tree")
    return anc, depth


def tree_attn(q, k, v, prefix_len, parent, num_nodes=None, *, scale=None,
              block_table=None, block_size=16):
    """Tree-masked attention by definition.

    q [B,N_max,Hq,D]; contiguous cache k,v [B,Hkv,S_cap,D], or paged
    [num_blocks,Hkv,block_size,D] with block_table [B,max_blocks].
    Returns (o [B,N_max,Hq,D] float64, lse [B,Hq,N_max] float64).
    """
    dt = _dtype_code(q)
    assert _dtype_code(k) == dt and _dtype_code(v) == dt
    B, N_max, Hq, D = q.shape
    Hkv = k.shape[1]
    assert q.strides[3] == q.itemsize and k.strides[3] == k.itemsize
    assert k.shape == v.shape and k.strides == v.strides
    qs = _estrides(q)
    ks = _estrides(k)
    prefix_len = _i32(prefix_len)
    parent = _i32(parent).reshape(B, N_max)
    nn = None if num_nodes is None else _i32(num_nodes)
    bt = None
    max_blocks = 0
    if block_table is not None:
        bt = _i32(block_table)
        max_blocks = bt.shape[1]
        assert k.shape[2] == block_size
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    o = np.zeros((B, N_max, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq, N_max), dtype=np.float64)
    I64 = ctypes.c_int64
    rc = _load().oracle_tree_attn(
        ctypes.c_int(dt), ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        ctypes.c_int(D), ctypes.c_int(N_max), ctypes.c_double(scale),
        _p(q), I64(qs[0]), I64(qs[1]), I64(qs[2]),
        _p(k), _p(v), I64(ks[0]), I64(ks[1]), I64(ks[2]),
        _p(bt), ctypes.c_int(block_size), ctypes.c_int(max_blocks),
        _p(prefix_len), _p(nn), _p(parent), _p(o), _p(lse))
    if rc:
        raise ValueError(f"oracle_tree_attn failed with status {rc}")
    return o, lse


def node_argmax(logits, num_nodes=None):
    """logits [B,N_max,V] (uint16 bf16 bits or float32) -> amax [B,N_max] int32."""
    dt = _dtype_code(logits)
    B, N_max, V = logits.shape
    assert logits.strides[2] == logits.itemsize
    st = _estrides(logits)
    nn = None if num_nodes is None else _i32(num_nodes)
    amax = np.zeros((B, N_max), dtype=np.int32)
    _load().oracle_node_argmax(
        ctypes.c_int(dt), ctypes.c_int(B), ctypes.c_int(N_max), ctypes.c_int(V),
        _p(logits), ctypes.c_int64(st[0]), ctypes.c_int64(st[1]), _p(nn), _p(amax))
    return amax


def head_argmax(hidden, W, num_nodes=None):
    """hidden [B,N_max,E], W [V,E] (uint16 bf16 bits or float32, same type).  Returns
    (amax [B,N_max] int32, max_logit [B,N_max] float64, gap [B,N_max] float64, second [B,N_max] int32)."""
    dt = _dtype_code(hidden)
    assert _dtype_code(W) == dt
    B, N_max, E = hidden.shape
    V = W.shape[0]
    assert W.shape[1] == E and hidden.strides[2] == hidden.itemsize and W.strides[1] == W.itemsize
    hs, ws = _estrides(hidden), _estrides(W)
    nn = None if num_nodes is None else _i32(num_nodes)
    amax = np.zeros((B, N_max), dtype=np.int32)
    mx = np.zeros((B, N_max), dtype=np.float64)
    gap = np.zeros((B, N_max), dtype=np.float64)
    second = np.zeros((B, N_max), dtype=np.int32)
    I64 = ctypes.c_int64
    _load().oracle_head_argmax(ctypes.c_int(dt), ctypes.c_int(B), ctypes.c_int(N_max), ctypes.c_int(E),
                               ctypes.c_int(V), _p(hidden), I64(hs[0]), I64(hs[1]), _p(W), I64(ws[0]), _p(nn),
                               _p(amax), _p(mx), _p(gap), _p(second))
    return amax, mx, gap, second


def tree_accept(parent, draft_tok, amax, num_nodes=None, path_cap=8):
    """Returns (accept_len [B], path [B,path_cap], bonus_tok [B], committed_tok [B,path_cap])."""
    parent = _i32(parent)
    B, N_max = parent.shape
    draft_tok = _i32(draft_tok).reshape(B, N_max)
    amax = _i32(amax).reshape(B, N_max)
    nn = None if num_nodes is None else _i32(num_nodes)
    accept_len = np.zeros(B, dtype=np.int32)
    path = np.zeros((B, path_cap), dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    committed = np.zeros((B, path_cap), dtype=np.int32)
    rc = _load().oracle_tree_accept(
        ctypes.c_int(B), ctypes.c_int(N_max), ctypes.c_int(path_cap),
        _p(parent), _p(draft_tok), _p(amax), _p(nn),
        _p(accept_len), _p(path), _p(bonus), _p(committed))
    if rc:
        raise ValueError(f"oracle_tree_accept failed with status {rc}")
    return accept_len, path, bonus, committed


def tree_accept_sample(parent, draft_tok, logits, u_accept, u_bonus, *, temperature=1.0, num_nodes=None,
                       path_cap=8):
    """Sampling-based acceptance.  logits [B,N_max,V] (uint16 bf16 bits or float32), u_accept [B,N_max] and
    u_bonus [B] float32 in [0,1).  Returns (accept_len, path, bonus_tok, committed_tok, info) where info holds
    margin_accept [B], margin_bonus [B] (float64) and bonus_alt [B] (see the C function)."""
    parent = _i32(parent)
    B, N_max = parent.shape
    draft_tok = _i32(draft_tok).reshape(B, N_max)
    dt = _dtype_code(logits)
    assert logits.shape[:2] == (B, N_max) and logits.strides[2] == logits.itemsize
    V = logits.shape[2]
    st = _estrides(logits)
    nn = None if num_nodes is None else _i32(num_nodes)
    ua = np.ascontiguousarray(u_accept, dtype=np.float32).reshape(B, N_max)
    ub = np.ascontiguousarray(u_bonus, dtype=np.float32).reshape(B)
    accept_len = np.zeros(B, dtype=np.int32)
    path = np.zeros((B, path_cap), dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    committed = np.zeros((B, path_cap), dtype=np.int32)
    margin_accept = np.zeros(B, dtype=np.float64)
    margin_bonus = np.zeros(B, dtype=np.float64)
    bonus_alt = np.zeros(B, dtype=np.int32)
    rc = _load().oracle_tree_accept_sample(
        ctypes.c_int(dt), ctypes.c_int(B), ctypes.c_int(N_max), ctypes.c_int(V), ctypes.c_int(path_cap),
        _p(parent), _p(draft_tok), _p(logits), ctypes.c_int64(st[0]), ctypes.c_int64(st[1]), _p(nn),
        ctypes.c_double(temperature), _p(ua), _p(ub),
        _p(accept_len), _p(path), _p(bonus), _p(committed), _p(margin_accept), _p(margin_bonus), _p(bonus_alt))
    if rc:
        raise ValueError(f"oracle_tree_accept_sample failed with status {rc}")
    return accept_len, path, bonus, committed, dict(margin_accept=margin_accept, margin_bonus=margin_bonus,
                                                    bonus_alt=bonus_alt)


def kv_compact(k, v, prefix_len, path, accept_len, *, block_table=None, block_size=16):
    """In-place compaction of k, v [L, ...cache dims...] (see tree_attn for the
    per-layer layouts).  Returns (new_prefix_len [B], moved_idx [B,path_cap,2])."""
    assert k.dtype == v.dtype and k.shape == v.shape and k.strides == v.strides
    assert k.flags.writeable and v.flags.writeable
    L = k.shape[0]
    Hkv, D = k.shape[2], k.shape[4]
    st = _estrides(k)
    prefix_len = _i32(prefix_len)
    B = prefix_len.shape[0]
    path = _i32(path).reshape(B, -1)
    path_cap = path.shape[1]
    accept_len = _i32(accept_len)
    bt = None
    max_blocks = 0
    if block_table is not None:
        bt = _i32(block_table)
        max_blocks = bt.shape[1]
    new_prefix = np.zeros(B, dtype=np.int32)
    moved = np.zeros((B, path_cap, 2), dtype=np.int32)
    I64 = ctypes.c_int64
    rc = _load().oracle_kv_compact(
        ctypes.c_int(L), ctypes.c_int(B), ctypes.c_int(Hkv), ctypes.c_int(D),
        ctypes.c_int(k.itemsize), _p(k), _p(v), I64(st[0]),
        I64(st[1]), I64(st[2]), I64(st[3]),
        _p(bt), ctypes.c_int(block_size), ctypes.c_int(max_blocks),
        _p(prefix_len), _p(path), ctypes.c_int(path_cap), _p(accept_len),
        _p(new_prefix), _p(moved))
    if rc:
        raise ValueError(f"oracle_kv_compact failed with status {rc}")
    return new_prefix, moved


# ---- draft side: growth of the token tree (Sec. 4.1: Top-K 10, 60 tokens, depth 7) ----------------

def topk_logprob(logits, K, cum=None):
    """logits [R,V] (uint16 bf16 bits or float32), cum [R] float64 or None.
    Returns (score [R,K] float64, token [R,K] int32, lse [R] float64)."""
    dt = _dtype_code(logits)
    R, V = logits.shape
    assert logits.strides[1] == logits.itemsize
    c = None if cum is None else np.ascontiguousarray(cum, dtype=np.float64).reshape(R)
    score = np.zeros((R, K), dtype=np.float64)
    token = np.zeros((R, K), dtype=np.int32)
    lse = np.zeros(R, dtype=np.float64)
    rc = _load().oracle_topk_logprob(
        ctypes.c_int(dt), ctypes.c_int(R), ctypes.c_int(V), ctypes.c_int(K), _p(logits),
        ctypes.c_int64(_estrides(logits)[0]), _p(c), _p(score), _p(token), _p(lse))
    if rc:
        raise ValueError(f"oracle_topk_logprob failed with status {rc}")
    return score, token, lse


def tree_select(score, M, num_cand=None):
    """score [B,C] float32.  Returns (sel [B,M] int32, -1 padded; count [B]; gap [B] float64)."""
    score = np.ascontiguousarray(score, dtype=np.float32)
    B, C = score.shape
    nc = None if num_cand is None else _i32(num_cand)
    sel = np.zeros((B, M), dtype=np.int32)
    count = np.zeros(B, dtype=np.int32)
    gap = np.zeros(B, dtype=np.float64)
    _load().oracle_tree_select(ctypes.c_int(B), ctypes.c_int(C), ctypes.c_int(M), _p(score), _p(nc),
                               _p(sel), _p(count), _p(gap))
    return sel, count, gap


def tree_finalize(cand_score, cand_parent, cand_token, root_token, N_max, num_cand=None):
    """Candidates [B,C] -> (parent [B,N_max], draft_tok [B,N_max], node_cand [B,N_max], num_nodes [B],
    gap [B] float64)."""
    cand_score = np.ascontiguousarray(cand_score, dtype=np.float32)
    B, C = cand_score.shape
    cp = _i32(cand_parent).reshape(B, C)
    ct = _i32(cand_token).reshape(B, C)
    rt = _i32(root_token).reshape(B)
    nc = None if num_cand is None else _i32(num_cand)
    parent = np.zeros((B, N_max), dtype=np.int32)
    tok = np.zeros((B, N_max), dtype=np.int32)
    node_cand = np.zeros((B, N_max), dtype=np.int32)
    num_nodes = np.zeros(B, dtype=np.int32)
    gap = np.zeros(B, dtype=np.float64)
    rc = _load().oracle_tree_finalize(
        ctypes.c_int(B), ctypes.c_int(C), ctypes.c_int(N_max), _p(cand_score), _p(cp), _p(ct), _p(nc), _p(rt),
        _p(parent), _p(tok), _p(node_cand), _p(num_nodes), _p(gap))
    if rc:
        raise ValueError(f"oracle_tree_finalize failed with status {rc}")
    return parent, tok, node_cand, num_nodes, gap


def grow_tree(level_logits, root_token, *, K=10, width=10, N_max=60):
    """Whole growth of one batch of draft trees from the draft model's logits.

    level_logits[0] is [B,1,V] (the root's next-token logits); level_logits[d], d >= 1, is
    [B,rows_d,V] with rows_d = min(width, candidates made by level d-1): row r belongs to the r-th
    node chosen for expansion at depth d (chosen nodes are listed in increasing candidate index).
    Level d expands its nodes by their Top-K tokens; a candidate's value is the sum of the
    log-probabilities on its root path, kept as float32 (the stored number every later choice is
    taken on); the `width` most valuable new candidates are expanded next; in the end the
    N_max - 1 most valuable candidates of all levels form the tree.

    Returns a dict: cand_score/cand_parent/cand_token [B,C], level_sel (list of [B,rows_d] global
    candidate indices), level_gap (list of [B]), and the outputs of tree_finalize.
    """
    depth = len(level_logits)
    B = level_logits[0].shape[0]
    V = level_logits[0].shape[2]
    C = sum(lg.shape[1] * K for lg in level_logits)
    cand_score = np.zeros((B, C), dtype=np.float32)
    cand_parent = np.full((B, C), -1, dtype=np.int32)
    cand_token = np.zeros((B, C), dtype=np.int32)
    level_sel, level_gap = [], []
    base, count = 0, 0                       # candidate range created by the previous level
    for d in range(depth):
        lg = level_logits[d]
        rows = lg.shape[1]
        if d == 0:
            assert rows == 1
            cum = np.zeros((B, 1), dtype=np.float64)
            par = np.full((B, 1), -1, dtype=np.int32)
            new_base = 0
        else:
            assert rows == min(width, count)
            sel, cnt, gap = tree_select(cand_score[:, base:base + count], rows)
            assert np.all(cnt == rows)
            sel = sel + base
            level_sel.append(sel)
            level_gap.append(gap)
            cum = np.take_along_axis(cand_score, sel, axis=1).astype(np.float64)
            par = sel
            new_base = base + count
        sc, tk, _ = topk_logprob(np.ascontiguousarray(lg).reshape(B * rows, V), K, cum.reshape(-1))
        n_new = rows * K
        cand_score[:, new_base:new_base + n_new] = sc.reshape(B, n_new).astype(np.float32)
        cand_token[:, new_base:new_base + n_new] = tk.reshape(B, n_new)
        cand_parent[:, new_base:new_base + n_new] = np.repeat(par, K, axis=1)
        base, count = new_base, n_new
    parent, tok, node_cand, num_nodes, gap = tree_finalize(cand_score, cand_parent, cand_token, root_token, N_max)
    return dict(cand_score=cand_score, cand_parent=cand_parent, cand_token=cand_token, level_sel=level_sel,
                level_gap=level_gap, parent=parent, draft_tok=tok, node_cand=node_cand, num_nodes=num_nodes,
                final_gap=gap)


# ---- parameter-free visual token compressors (draft side) ------------------------------------------

def visual_pool(x, ratio, num_tokens=None):
    """x [B,T,E] (uint16 bf16 bits or float32) -> (y [B,ceil(T/ratio),E] float64, out_tokens [B])."""
    dt = _dtype_code(x)
    B, T, E = x.shape
    assert x.strides[2] == x.itemsize
    st = _estrides(x)
    nt = None if num_tokens is None else _i32(num_tokens)
    Tp = (T + ratio - 1) // ratio
    y = np.zeros((B, Tp, E), dtype=np.float64)
    out_tokens = np.zeros(B, dtype=np.int32)
    rc = _load().oracle_visual_pool(ctypes.c_int(dt), ctypes.c_int(B), ctypes.c_int(T), ctypes.c_int(E),
                                    ctypes.c_int(ratio), _p(x), ctypes.c_int64(st[0]), ctypes.c_int64(st[1]),
                                    _p(nt), _p(y), _p(out_tokens))
    if rc:
        raise ValueError(f"oracle_visual_pool failed with status {rc}")
    return y, out_tokens


def visual_prune(x, keep):
    """x [B,T,E], keep [B,T_keep] int32 (-1 = padding) -> y [B,T_keep,E] of x's dtype (padding rows zero)."""
    B, T, E = x.shape
    assert x.strides[2] == x.itemsize
    st = _estrides(x)
    keep = _i32(keep).reshape(B, -1)
    y = np.zeros((B, keep.shape[1], E), dtype=x.dtype)
    rc = _load().oracle_visual_prune(ctypes.c_int(x.itemsize), ctypes.c_int(B), ctypes.c_int(T),
                                     ctypes.c_int(keep.shape[1]), ctypes.c_int(E), _p(x), ctypes.c_int64(st[0]),
                                     ctypes.c_int64(st[1]), _p(keep), _p(y))
    if rc:
        raise ValueError(f"oracle_visual_prune failed with status {rc}")
    return y
