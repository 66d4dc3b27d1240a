"""Helpers of the GPU parity tests: numpy <-> device tensors and oracle comparisons."""
from __future__ import annotations

import numpy as np
import torch

import workloads as W

# Tolerances of the attention output against the fp64 oracle:
#   bf16 tensors: max-abs 2e-2, mean-abs 2e-3 (inputs, P and the output are rounded to bf16,
#                 8 mantissa bits; outputs are O(1) convex combinations of N(0,1) rows)
#   fp32 tensors: max-abs 1e-5 (fp32 dot products and exp over <= a few thousand keys)
TOL = {"bf16": (2e-2, 2e-3), "f32": (1e-5, 1e-5)}


def to_dev(a: np.ndarray | None):
    """uint16 arrays are bf16 bit patterns; float32/int32 pass through."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.detach().cpu().numpy()


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def assert_attn_close(got: np.ndarray, ref: np.ndarray, dtype: str, what: str = ""):
    max_tol, mean_tol = TOL[dtype]
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - ref)
    assert err.max() <= max_tol, f"{what}: max-abs {err.max():.3e} > {max_tol}"
    assert err.mean() <= mean_tol, f"{what}: mean-abs {err.mean():.3e} > {mean_tol}"


def valid_rows_mask(B, N_max, num_nodes):
    m = np.zeros((B, N_max), dtype=bool)
    for b in range(B):
        m[b, :(N_max if num_nodes is None else int(num_nodes[b]))] = True
    return m


def random_case(seed, dtype, B, Hq, Hkv, D, N_max, P_list, *, num_nodes=None, paged=False,
                depth=6, cap_extra=7, tree="random"):
    """Small random attention problem with poisoned unused slots."""
    rng = np.random.default_rng(seed)
    nn = np.full(B, N_max, dtype=np.int32) if num_nodes is None else np.array(num_nodes, dtype=np.int32)
    P = np.array(P_list, dtype=np.int32)
    S = P + nn
    q = W.normal(rng, (B, N_max, Hq, D), 1.0, dtype)
    parent = np.stack([W.chain_tree(N_max) if tree == "chain" else W.random_tree(rng, N_max, depth)
                       for _ in range(B)])
    poison = W.NAN_BITS_BF16 if dtype == "bf16" else np.float32(np.nan)
    for b in range(B):                                   # query rows past the node count are never to matter
        q[b, nn[b]:] = poison
    if not paged:
        cap = W.round_up(int(S.max()) + cap_extra, 8)
        k = W.normal(rng, (B, Hkv, cap, D), 1.0, dtype)
        v = W.normal(rng, (B, Hkv, cap, D), 1.0, dtype)
        for b in range(B):
            k[b, :, S[b]:] = poison
            v[b, :, S[b]:] = poison
        table = None
    else:
        bs = 16
        bpr = W.round_up(int(S.max()), bs) // bs + 1
        table, nb = W.block_table(rng, B, bpr, spare=0.25)
        k = W.normal(rng, (nb, Hkv, bs, D), 1.0, dtype)
        v = W.normal(rng, (nb, Hkv, bs, D), 1.0, dtype)
        used = np.zeros(nb, dtype=bool)
        used[table.reshape(-1)] = True
        k[~used] = poison
        v[~used] = poison
        for b in range(B):
            for slot in range(int(S[b]), bpr * bs):
                k[table[b, slot // bs], :, slot % bs] = poison
                v[table[b, slot // bs], :, slot % bs] = poison
    return dict(q=q, k=k, v=v, prefix_len=P, num_nodes=None if num_nodes is None else nn,
                parent=parent, block_table=table, dtype=dtype)
