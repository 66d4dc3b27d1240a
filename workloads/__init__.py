"""Seeded synthetic inputs for the tree-verification step.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It holds none of the method's arithmetic (no attention, no vocab
argmax, no acceptance walk, no compaction): it only draws random tensors,
tree shapes, token ids and block tables with the shapes of the paper's
workloads (Sec. 4.1: LLaVA-1.5/1.6 7B/13B targets, batch 1, draft tree with
Top-K 10, 60 tokens, depth 7) and rounds them to the storage type.

They stand in for the paper's LLaVA-suite / MMMU requests, whose items are not
used here: only tensor shapes and the tree hyper-parameters are taken.

bf16 tensors are produced as ``uint16`` bit patterns (numpy has no bf16).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 11815 * 1000
NAN_BITS_BF16 = np.uint16(0x7FC1)


# --------------------------------------------------------------------------
# storage-type helpers
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), return uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = NAN_BITS_BF16
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(rng: np.random.Generator, shape, sigma: float, dtype: str) -> np.ndarray:
    """N(0, sigma^2) draws in the storage type: 'bf16' -> uint16 bits, 'f32' -> float32."""
    x = rng.standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def as_f64(a: np.ndarray) -> np.ndarray:
    """Stored tensor (uint16 bf16 bits or float32) -> float64 values."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------
# tree shapes
# --------------------------------------------------------------------------
def chain_tree(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int32)


def random_tree(rng: np.random.Generator, n: int, max_depth: int) -> np.ndarray:
    """parent[i] uniform in [0,i), redrawn while the node would exceed max_depth."""
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        while True:
            p = int(rng.integers(0, i))
            if depth[p] + 1 <= max_depth:
                break
        parent[i] = p
        depth[i] = depth[p] + 1
    return parent


def eagle_tree(rng: np.random.Generator, n_nodes: int = 60, depth: int = 6, topk: int = 10):
    """EAGLE-2-shaped tree: level-by-level top-k expansion, then keep the best n_nodes.

    Every expanded node gets `topk` children whose probabilities are the sorted
    softmax of `topk` N(0,1.5) draws; a node's score is the product of the
    probabilities on its root path; per level the `topk` best new nodes are
    expanded; finally the root, the best node of the last level with its root
    path (so the stated depth is reached) and the best-scoring remaining nodes are kept and
    renumbered by (depth, -score) so that parent[i] < i.

    Returns (parent [n_nodes] int32, score [n_nodes] float64, rank [n_nodes]
    int32 = position of the node among its kept siblings, 0 = most likely).
    """
    par, score, dep = [-1], [1.0], [0]
    frontier = [0]
    for level in range(1, depth + 1):
        new = []
        for node in frontier:
            z = rng.normal(0.0, 1.5, size=topk)
            pr = np.exp(z - z.max())
            pr = np.sort(pr / pr.sum())[::-1]
            for c in range(topk):
                par.append(node)
                score.append(score[node] * float(pr[c]))
                dep.append(level)
                new.append(len(par) - 1)
        new.sort(key=lambda t: -score[t])
        frontier = new[:topk]
    par = np.array(par)
    score = np.array(score)
    dep = np.array(dep)
    keep = {0}
    deepest = np.nonzero(dep == depth)[0]
    t = int(deepest[np.argmax(score[deepest])])     # best node of the last level and its root path,
    while t != -1:                                  # so that the stated depth is reached
        keep.add(t)
        t = int(par[t])
    for t in np.argsort(-score, kind="stable"):
        if len(keep) >= n_nodes:
            break
        keep.add(int(t))
    kept = sorted(keep, key=lambda t: (dep[t], -score[t], t))
    assert len(kept) == n_nodes
    new_id = {old: i for i, old in enumerate(kept)}
    parent = np.array([-1 if par[t] < 0 else new_id[int(par[t])] for t in kept], dtype=np.int32)
    assert all(parent[i] < i for i in range(1, n_nodes)), "kept set must be ancestor-closed"
    sc = score[kept]
    rank = np.zeros(n_nodes, dtype=np.int32)
    for p in range(n_nodes):
        kids = [i for i in range(1, n_nodes) if parent[i] == p]
        for r, i in enumerate(sorted(kids, key=lambda i: -sc[i])):
            rank[i] = r
    return parent, sc, rank


def tree_depths(parent: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


# --------------------------------------------------------------------------
# logits and draft tokens
# --------------------------------------------------------------------------
def planted_logits(rng: np.random.Generator, rows: int, V: int, sigma: float, dtype: str):
    """i.i.d. N(0, sigma^2) logits rows whose largest draw sits at a known token.

    Each row is a sorted i.i.d. sample scattered through a uniformly random
    permutation of the vocabulary, which is again an i.i.d. sample; the token
    that received the largest draw is returned as `top_tok` without scanning
    the row.  After rounding to bf16 the largest value can tie with others, so
    `top_tok` is the *intended* greedy token, not a computed argmax.
    """
    logits = np.empty((rows, V), dtype=np.uint16 if dtype == "bf16" else np.float32)
    top_tok = np.empty(rows, dtype=np.int32)
    for r in range(rows):
        vals = np.sort(rng.standard_normal(V, dtype=np.float32) * np.float32(sigma))[::-1]
        perm = rng.permutation(V)
        row = np.empty(V, dtype=np.float32)
        row[perm] = vals
        logits[r] = f32_to_bf16_bits(row) if dtype == "bf16" else row
        top_tok[r] = perm[0]
    return logits, top_tok


def draft_tokens_topk(rng: np.random.Generator, parent, rank, top_tok, V: int, alpha: float):
    """Sibling-distinct draft tokens; with probability alpha the most likely kept
    child of a node carries that node's intended greedy token."""
    n = len(parent)
    tok = np.zeros(n, dtype=np.int32)
    tok[0] = int(rng.integers(0, V))
    for p in range(n):
        kids = [i for i in range(1, n) if parent[i] == p]
        if not kids:
            continue
        hit = rng.random() < alpha
        pool = rng.choice(V - 1, size=len(kids), replace=False)
        pool = np.where(pool >= top_tok[p], pool + 1, pool)      # all != top_tok[p], distinct
        for i, t in zip(kids, pool):
            tok[i] = int(t)
        if hit:
            first = [i for i in kids if rank[i] == 0][0]
            tok[first] = int(top_tok[p])
    return tok


def draft_tokens_uniform(rng: np.random.Generator, parent, top_tok, V: int, p_match: float):
    """Uniform tokens; each non-root node independently copies its parent's intended
    greedy token with probability p_match (equal sibling tokens can occur)."""
    n = len(parent)
    tok = rng.integers(0, V, size=n).astype(np.int32)
    for i in range(1, n):
        if rng.random() < p_match:
            tok[i] = int(top_tok[parent[i]])
    return tok


# --------------------------------------------------------------------------
# paged cache
# --------------------------------------------------------------------------
def block_table(rng: np.random.Generator, B: int, blocks_per_req: int, spare: float = 0.1):
    """Seeded random assignment of physical blocks: a permutation of a pool with
    `spare` extra blocks.  Returns (table [B, blocks_per_req] int32, num_blocks)."""
    need = B * blocks_per_req
    num_blocks = need + max(1, int(np.ceil(need * spare)))
    perm = rng.permutation(num_blocks)[:need]
    return perm.reshape(B, blocks_per_req).astype(np.int32), num_blocks


# --------------------------------------------------------------------------
# the five workload configurations
# --------------------------------------------------------------------------
@dataclass
class Config:
    name: str
    index: int
    dtype: str            # 'bf16' | 'f32'
    L: int
    H: int
    D: int
    B: int
    N: int                # tree nodes per request (root included) == N_max
    depth: int
    V: int
    sigma_logits: float
    paged: bool = False
    block_size: int = 16
    prefix: tuple = ()    # fixed per-request committed prefix lengths, or () if drawn
    tree: str = "eagle"   # 'eagle' | 'random'
    alpha: float = 0.75
    tree_salt: int = 0    # added to the tree/logit seed; picks which seeded draw the config uses
    note: str = ""
    extra: dict = field(default_factory=dict)


CONFIGS = {
    "C1": Config("C1", 1, "f32", 1, 4, 64, 1, 8, 3, 1000, 1.0, prefix=(64,), tree="random",
                 alpha=0.5, note="tiny fp32 plumbing case"),
    "C2": Config("C2", 2, "bf16", 32, 32, 128, 1, 60, 6, 32000, 2.0, prefix=(576 + 64 + 128,), tree_salt=5,
                 note="LLaVA-1.5-7B-shaped, 576 visual + 64 text + 128 generated"),
    "C3": Config("C3", 3, "bf16", 32, 32, 128, 1, 60, 6, 32000, 2.0, prefix=(2880 + 128 + 256,), tree_salt=3,
                 note="LLaVA-1.6-7B anyres-shaped, 2880 visual + 128 text + 256 generated"),
    "C4": Config("C4", 4, "bf16", 32, 32, 128, 8, 60, 6, 32000, 2.0,
                 note="compressed-visual variable-length batch",
                 extra={"visual": (64, 144, 288, 720), "text": (32, 256)}),
    "C5": Config("C5", 5, "bf16", 40, 40, 128, 4, 60, 7, 32000, 2.0, paged=True,
                 prefix=(8 * 576 + 256,) * 4,
                 note="multi-frame 13B-shaped, 8x576 visual + 256 text/generated, paged cache"),
}


def config_seed(cfg: Config, layer: int = 0, stream: int = 0) -> int:
    return SEED_BASE + 100 * cfg.index + layer + 1_000_000 * stream


def prefix_lengths(cfg: Config) -> np.ndarray:
    if cfg.prefix:
        return np.array(cfg.prefix, dtype=np.int32)
    rng = np.random.default_rng(config_seed(cfg, 0, stream=7))
    vis = rng.choice(np.array(cfg.extra["visual"]), size=cfg.B)
    lo, hi = cfg.extra["text"]
    txt = rng.integers(lo, hi + 1, size=cfg.B)
    return (vis + txt).astype(np.int32)


def round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


@dataclass
class TreeBatch:
    parent: np.ndarray      # [B, N] int32
    draft_tok: np.ndarray   # [B, N] int32
    logits: np.ndarray      # [B, N, V] storage type
    top_tok: np.ndarray     # [B, N] intended greedy token per node (by construction)


def make_trees(cfg: Config) -> TreeBatch:
    """Trees, draft tokens and target logits of one verify step."""
    rng = np.random.default_rng(config_seed(cfg, cfg.tree_salt, stream=1))
    parents, toks = [], []
    logits, top = planted_logits(rng, cfg.B * cfg.N, cfg.V, cfg.sigma_logits, cfg.dtype)
    logits = logits.reshape(cfg.B, cfg.N, cfg.V)
    top = top.reshape(cfg.B, cfg.N)
    for b in range(cfg.B):
        if cfg.tree == "eagle":
            parent, _, rank = eagle_tree(rng, cfg.N, cfg.depth, 10)
            tok = draft_tokens_topk(rng, parent, rank, top[b], cfg.V, cfg.alpha)
        else:
            parent = random_tree(rng, cfg.N, cfg.depth)
            tok = draft_tokens_uniform(rng, parent, top[b], cfg.V, cfg.alpha)
        parents.append(parent)
        toks.append(tok)
    return TreeBatch(np.stack(parents), np.stack(toks), logits, top)


@dataclass
class AttnLayer:
    q: np.ndarray             # [B, N, H, D]
    k: np.ndarray             # contiguous [B, H, S_cap, D] or paged [num_blocks, H, bs, D]
    v: np.ndarray
    prefix_len: np.ndarray    # [B] int32
    block_table: np.ndarray | None
    S_cap: int


def make_attn_layer(cfg: Config, layer: int, *, heads: int | None = None,
                    poison_tail: bool = True) -> AttnLayer:
    """q and the K/V cache of one layer (tree rows already written into slots
    [P_b, P_b+N)).  `heads` < cfg.H draws a narrower layer of the same shape per head
    (for oracle-sized samples).  Slots past P_b+N hold NaN patterns when poison_tail."""
    H = heads or cfg.H
    rng = np.random.default_rng(config_seed(cfg, layer, stream=2))
    P = prefix_lengths(cfg)
    S = P + cfg.N
    q = normal(rng, (cfg.B, cfg.N, H, cfg.D), 1.0, cfg.dtype)
    poison = NAN_BITS_BF16 if cfg.dtype == "bf16" else np.float32(np.nan)
    if not cfg.paged:
        S_cap = round_up(int(S.max()), 16)
        k = normal(rng, (cfg.B, H, S_cap, cfg.D), 1.0, cfg.dtype)
        v = normal(rng, (cfg.B, H, S_cap, cfg.D), 1.0, cfg.dtype)
        if poison_tail:
            for b in range(cfg.B):
                k[b, :, S[b]:, :] = poison
                v[b, :, S[b]:, :] = poison
        return AttnLayer(q, k, v, P, None, S_cap)
    bs = cfg.block_size
    blocks_per_req = round_up(int(S.max()), bs) // bs
    trng = np.random.default_rng(config_seed(cfg, 0, stream=3))   # one table for all layers
    table, num_blocks = block_table(trng, cfg.B, blocks_per_req)
    k = normal(rng, (num_blocks, H, bs, cfg.D), 1.0, cfg.dtype)
    v = normal(rng, (num_blocks, H, bs, cfg.D), 1.0, cfg.dtype)
    if poison_tail:
        used = np.zeros(num_blocks, dtype=bool)
        used[table.reshape(-1)] = True
        k[~used] = poison
        v[~used] = poison
        for b in range(cfg.B):
            for slot in range(int(S[b]), blocks_per_req * bs):
                k[table[b, slot // bs], :, slot % bs, :] = poison
                v[table[b, slot // bs], :, slot % bs, :] = poison
    return AttnLayer(q, k, v, P, table, blocks_per_req * bs)


def kv_bytes_per_layer(cfg: Config) -> int:
    """Algorithmic K+V bytes one attention call must stream: sum_b (P_b+N) * H * D * 2 * E."""
    E = 2 if cfg.dtype == "bf16" else 4
    S = prefix_lengths(cfg).astype(np.int64) + cfg.N
    return int(S.sum()) * cfg.H * cfg.D * 2 * E
