"""Seeded synthetic inputs for the blended decoder-layer step.

This module only draws random numbers and lays out integer tables.  It holds
none of the layer's arithmetic and none of the scheduling arithmetic: both the
CPU oracle's tests and the HIP path's tests take their inputs from here, and
neither implementation is imported here.

What the inputs stand in for (BlendServe, Section 6.2 and Appendix A.3): short
prompt-heavy API requests become the prefill segments, long-output requests
become the long decode contexts, and benchmark-style shared system prompts
become the prefix groups whose KV pages are referenced by every member.

Draw order (fixed, so that a seed names one input):
  structure stream  rng([seed, 1]):  lengths, then the physical page permutation
  tensor stream     rng([seed, 2]):  w_qkv, w_o, w_gate, w_up, w_down, x, K pool, V pool
Weights ~ N(0, 0.02^2), x ~ N(0, 1), cached K and V ~ N(0, 1); every tensor is
rounded once to bfloat16 (round-to-nearest-even) and both sides receive those
same values.  RMSNorm gains are 1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

PAGE = 16


# ----------------------------------------------------------------------------
# bfloat16 <-> float32 bit conversions (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bfloat16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# ----------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerShape:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    page_size: int = PAGE
    rms_eps: float = 1e-5
    rope_theta: float = 500000.0

    @property
    def n_qkv(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def matrix_params(self) -> int:
        d, f = self.d_model, self.d_ffn
        return d * self.n_qkv + self.n_q_heads * self.head_dim * d + 3 * d * f

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2


TINY = LayerShape(256, 4, 2, 64, 688)
LLAMA3_8B = LayerShape(4096, 32, 8, 128, 14336)
LLAMA3_70B = LayerShape(8192, 64, 8, 128, 28672)


# ----------------------------------------------------------------------------
# batch descriptor
# ----------------------------------------------------------------------------
@dataclass
class Batch:
    """Host-side description of one blended step (all arrays int32).

    Sequences [0, n_prefill) are prefill segments, the rest decode sequences
    with exactly one row each.  `kv_len[i]` is the attended length after this
    step's rows have been appended; rows of sequence i sit at positions
    kv_len[i]-q_len[i] .. kv_len[i]-1.  Token t of sequence i lives in physical
    page page_ids[page_start[i] + t // page_size], slot t % page_size.  A prefix
    node is a run of pages shared by the contiguous run of sequences
    [node_seq_first, node_seq_first + node_seq_count); nodes are listed in DFS
    pre-order and a child's pages follow its parent's in every member's table.
    """
    page_size: int
    n_seq: int
    n_prefill: int
    n_rows: int
    row_start: np.ndarray
    kv_len: np.ndarray
    page_start: np.ndarray
    page_ids: np.ndarray
    n_nodes: int
    node_parent: np.ndarray
    node_page_start: np.ndarray
    node_page_ids: np.ndarray
    node_seq_first: np.ndarray
    node_seq_count: np.ndarray
    seq_leaf_node: np.ndarray
    n_pages: int = 0  # size of the physical pool these ids index

    def q_len(self) -> np.ndarray:
        return np.diff(self.row_start)

    def copy(self) -> "Batch":
        kw = {}
        for k, v in self.__dict__.items():
            kw[k] = v.copy() if isinstance(v, np.ndarray) else v
        return Batch(**kw)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64).astype(np.int32))


def assemble_batch(page_size: int,
                   seqs: Sequence[Tuple[int, int, int]],
                   n_prefill: int,
                   nodes: Sequence[Tuple[int, int]],
                   rng: Optional[np.random.Generator],
                   spare_pages: int = 8) -> Batch:
    """Lay out page tables for a batch.

    seqs:  (q_len, kv_len, leaf_node) per sequence, prefill segments first;
           members of a node must be contiguous and children follow parents.
           A prefill segment that names a node only borrows the pages of that
           node's root path as its cached prefix: it is not a member of the node
           (node members are decode sequences) and its seq_leaf_node is -1.
    nodes: (parent, n_pages) in DFS pre-order.
    Logical pages are numbered node pages first, then private pages, and mapped
    to physical ids by a random permutation of the pool (identity if rng is
    None).  `spare_pages` pool pages are referenced by nobody.
    """
    n_nodes = len(nodes)
    n_seq = len(seqs)
    parent = [p for p, _ in nodes]
    node_np = [n for _, n in nodes]
    depth_pages = [0] * n_nodes           # pages on the path above the node
    for i, (p, n) in enumerate(nodes):
        assert p < i, "nodes must be in DFS pre-order"
        depth_pages[i] = 0 if p < 0 else depth_pages[p] + node_np[p]
    node_page_start = np.zeros(n_nodes + 1, dtype=np.int64)
    node_page_start[1:] = np.cumsum(node_np)
    next_logical = int(node_page_start[-1])

    # membership runs
    first = [n_seq] * n_nodes
    last = [-1] * n_nodes
    for s, (_, _, leaf) in enumerate(seqs):
        nd = leaf if s >= n_prefill else -1
        while nd >= 0:
            first[nd] = min(first[nd], s)
            last[nd] = max(last[nd], s)
            nd = parent[nd]
    count = [max(0, last[i] - first[i] + 1) for i in range(n_nodes)]
    first = [first[i] if count[i] else 0 for i in range(n_nodes)]

    page_start = [0]
    logical: List[int] = []
    for s, (q_len, kv_len, leaf) in enumerate(seqs):
        assert q_len >= 1 and kv_len >= q_len
        path = []
        nd = leaf
        while nd >= 0:
            path.append(nd)
            nd = parent[nd]
        path.reverse()
        shared = 0
        for nd in path:
            lo = int(node_page_start[nd])
            logical.extend(range(lo, lo + node_np[nd]))
            shared += node_np[nd]
        assert shared * page_size <= kv_len - q_len, "appended rows must land in private pages"
        total = -(-kv_len // page_size)
        n_priv = total - shared
        logical.extend(range(next_logical, next_logical + n_priv))
        next_logical += n_priv
        page_start.append(len(logical))
    n_pages = next_logical + spare_pages
    perm = np.arange(n_pages) if rng is None else rng.permutation(n_pages)
    logical_arr = np.asarray(logical, dtype=np.int64)
    row_start = np.zeros(n_seq + 1, dtype=np.int64)
    row_start[1:] = np.cumsum([q for q, _, _ in seqs])
    return Batch(
        page_size=page_size, n_seq=n_seq, n_prefill=n_prefill, n_rows=int(row_start[-1]),
        row_start=_i32(row_start), kv_len=_i32([k for _, k, _ in seqs]),
        page_start=_i32(page_start),
        page_ids=_i32(perm[logical_arr] if len(logical) else []),
        n_nodes=n_nodes, node_parent=_i32(parent),
        node_page_start=_i32(node_page_start),
        node_page_ids=_i32(perm[np.arange(int(node_page_start[-1]))] if n_nodes else []),
        node_seq_first=_i32(first), node_seq_count=_i32(count),
        seq_leaf_node=_i32([(l if s >= n_prefill else -1) for s, (_, _, l) in enumerate(seqs)]),
        n_pages=int(n_pages))


def expand_batch(b: Batch) -> Tuple[Batch, np.ndarray]:
    """Physically unshared twin of a batch.

    Returns (batch with no nodes and a private copy of every page per sequence,
    src) where src[new_page] is the old physical page to copy the contents from
    (-1 for pages nobody references).  Used for the invariant that prefix-shared
    and expanded KV give the same output.
    """
    n_ref = int(b.page_start[-1])
    src = np.concatenate([b.page_ids.astype(np.int64), np.full(4, -1, dtype=np.int64)])
    e = b.copy()
    e.page_ids = _i32(np.arange(n_ref))
    e.n_nodes = 0
    e.node_parent = _i32([])
    e.node_page_start = _i32([0])
    e.node_page_ids = _i32([])
    e.node_seq_first = _i32([])
    e.node_seq_count = _i32([])
    e.seq_leaf_node = _i32(np.full(b.n_seq, -1))
    e.n_pages = n_ref + 4
    return e, src


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------
def batch_tiny(seed: int = 0) -> Batch:
    """2 prefill segments of 64 rows (no cache) + 8 decode sequences of context
    128 that all share one 96-token prefix (6 pages) and own 2 private pages."""
    rng = np.random.default_rng([seed, 1])
    seqs = [(64, 64, -1), (64, 64, -1)] + [(1, 128, 0)] * 8
    return assemble_batch(PAGE, seqs, 2, [(-1, 6)], rng)


def batch_decode_only(n_seq: int = 256, ctx: int = 1024, seed: int = 0) -> Batch:
    rng = np.random.default_rng([seed, 1])
    return assemble_batch(PAGE, [(1, ctx, -1)] * n_seq, 0, [], rng)


def batch_prefill_only(n_seg: int = 8, seg_len: int = 1024, seed: int = 0) -> Batch:
    rng = np.random.default_rng([seed, 1])
    return assemble_batch(PAGE, [(seg_len, seg_len, -1)] * n_seg, n_seg, [], rng)


def lognormal_contexts(rng: np.random.Generator, n: int, median: float = 1536.0,
                       sigma: float = 0.75, lo: int = 256, hi: int = 8192) -> np.ndarray:
    z = rng.standard_normal(n)
    return np.clip(np.rint(median * np.exp(sigma * z)), lo, hi).astype(np.int64)


def batch_blended_8b(seed: int = 0, n_groups: int = 32, per_group: int = 16,
                     prefix_tokens: int = 1024, n_seg: int = 4, seg_len: int = 512) -> Batch:
    """2048 prefill rows + 512 decode sequences with lognormal contexts in 32
    prefix groups.  A sequence shares min(prefix pages, (L-1)//16) whole pages of
    its group's prefix, so a group's prefix is a chain of nodes that members
    leave as their contexts run out (last token always private)."""
    rng = np.random.default_rng([seed, 1])
    ctx = lognormal_contexts(rng, n_groups * per_group)
    pp = prefix_tokens // PAGE
    seqs: List[Tuple[int, int, int]] = [(seg_len, seg_len, -1)] * n_seg
    nodes: List[Tuple[int, int]] = []
    for g in range(n_groups):
        L = ctx[g * per_group:(g + 1) * per_group]
        share = np.minimum(pp, (L - 1) // PAGE)
        order = np.argsort(-share, kind="stable")
        L, share = L[order], share[order]
        levels = sorted(set(int(s) for s in share))
        prev_end, prev_node = 0, -1
        node_of_level = {}
        for lv in levels:
            nodes.append((prev_node, lv - prev_end))
            prev_node = len(nodes) - 1
            node_of_level[lv] = prev_node
            prev_end = lv
        for i in range(per_group):
            seqs.append((1, int(L[i]), node_of_level[int(share[i])]))
    return assemble_batch(PAGE, seqs, n_seg, nodes, rng)


def batch_blended_70b(seed: int = 0, n_roots: int = 8, n_children: int = 8, per_child: int = 16,
                      root_tokens: int = 2048, child_tokens: int = 512,
                      n_seg: int = 8, seg_len: int = 512) -> Batch:
    """4096 prefill rows + 1024 decode sequences under a two-level prefix tree;
    private tails uniform in [16, 1024]."""
    rng = np.random.default_rng([seed, 1])
    tails = rng.integers(16, 1025, size=n_roots * n_children * per_child)
    seqs: List[Tuple[int, int, int]] = [(seg_len, seg_len, -1)] * n_seg
    nodes: List[Tuple[int, int]] = []
    t = 0
    for _ in range(n_roots):
        nodes.append((-1, root_tokens // PAGE))
        root = len(nodes) - 1
        for _ in range(n_children):
            nodes.append((root, child_tokens // PAGE))
            child = len(nodes) - 1
            for _ in range(per_child):
                seqs.append((1, root_tokens + child_tokens + int(tails[t]), child))
                t += 1
    return assemble_batch(PAGE, seqs, n_seg, nodes, rng)


def batch_random(seed: int, n_prefill: int = 3, n_decode: int = 9, max_q: int = 40,
                 max_ctx: int = 150, n_roots: int = 2, page_size: int = PAGE) -> Batch:
    """Small irregular batch for tests: a random two-level prefix forest, prefill
    chunks with and without cached (possibly shared) prefixes, ragged lengths,
    sequences outside every node."""
    rng = np.random.default_rng([seed, 1])
    nodes: List[Tuple[int, int]] = []
    leaves: List[int] = []
    for _ in range(n_roots):
        nodes.append((-1, int(rng.integers(1, 4))))
        root = len(nodes) - 1
        kids = int(rng.integers(0, 3))
        if kids == 0:
            leaves.append(root)
        for _ in range(kids):
            nodes.append((root, int(rng.integers(1, 3))))
            leaves.append(len(nodes) - 1)
        if kids and rng.random() < 0.5:
            leaves.append(root)  # some members stop at the root node
    parent = [p for p, _ in nodes]

    def shared_tokens(leaf: int) -> int:
        n, nd = 0, leaf
        while nd >= 0:
            n += nodes[nd][1]
            nd = parent[nd]
        return n * page_size

    def dfs_key(leaf: int) -> Tuple[int, ...]:
        path, nd = [], leaf
        while nd >= 0:
            path.append(nd)
            nd = parent[nd]
        return tuple(reversed(path))

    def draw(kind: str) -> Tuple[int, int, int]:
        leaf = -1 if rng.random() < 0.3 or not leaves else int(rng.choice(leaves))
        sh = shared_tokens(leaf) if leaf >= 0 else 0
        q = int(rng.integers(1, max_q + 1)) if kind == "p" else 1
        cached = sh + int(rng.integers(0, max_ctx))
        if kind == "p" and leaf < 0 and rng.random() < 0.5:
            cached = 0
        return (q, cached + q, leaf)

    def order(items):
        # members of a node contiguous, children grouped under parents: sort by DFS path,
        # sequences that stop at an inner node go before those of its children
        return sorted(items, key=lambda s: (0,) + dfs_key(s[2]) if s[2] >= 0 else (1,))

    pre = [draw("p") for _ in range(n_prefill)]   # prefill chunks borrow prefix pages, in any order
    dec = order([draw("d") for _ in range(n_decode)])
    return assemble_batch(page_size, pre + dec, n_prefill, nodes, rng)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
@dataclass
class Tensors:
    """float32 arrays hold bfloat16-representable values; pools are bf16 bits."""
    w_qkv: np.ndarray    # [d, (Hq+2Hkv)*dh]  columns: q heads, k heads, v heads
    w_o: np.ndarray      # [Hq*dh, d]
    w_gate: np.ndarray   # [d, F]
    w_up: np.ndarray     # [d, F]
    w_down: np.ndarray   # [F, d]
    g_attn: np.ndarray   # [d]
    g_ffn: np.ndarray    # [d]
    x: np.ndarray        # [T, d]
    k_pool: np.ndarray   # uint16 [n_pages, page, Hkv, dh]
    v_pool: np.ndarray   # uint16 [n_pages, page, Hkv, dh]


def _normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return round_to_bf16(a)


def _normal_bf16_bits(rng: np.random.Generator, shape) -> np.ndarray:
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(-1)
    step = 1 << 24
    for lo in range(0, flat.size, step):
        hi = min(flat.size, lo + step)
        flat[lo:hi] = f32_to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32))
    return out


def make_tensors(shape: LayerShape, batch: Batch, seed: int = 0,
                 gains: str = "ones") -> Tensors:
    rng = np.random.default_rng([seed, 2])
    d, f = shape.d_model, shape.d_ffn
    w_qkv = _normal_bf16(rng, (d, shape.n_qkv), 0.02)
    w_o = _normal_bf16(rng, (shape.n_q_heads * shape.head_dim, d), 0.02)
    w_gate = _normal_bf16(rng, (d, f), 0.02)
    w_up = _normal_bf16(rng, (d, f), 0.02)
    w_down = _normal_bf16(rng, (f, d), 0.02)
    x = _normal_bf16(rng, (batch.n_rows, d), 1.0)
    pool_shape = (batch.n_pages, shape.page_size, shape.n_kv_heads, shape.head_dim)
    k_pool = _normal_bf16_bits(rng, pool_shape)
    v_pool = _normal_bf16_bits(rng, pool_shape)
    if gains == "ones":
        g1 = np.ones(d, dtype=np.float32)
        g2 = np.ones(d, dtype=np.float32)
    else:  # non-trivial gains for tests of the norm path
        g1 = round_to_bf16(1.0 + 0.25 * rng.standard_normal(d, dtype=np.float32))
        g2 = round_to_bf16(1.0 + 0.25 * rng.standard_normal(d, dtype=np.float32))
    return Tensors(w_qkv, w_o, w_gate, w_up, w_down, g1, g2, x, k_pool, v_pool)


# ----------------------------------------------------------------------------
# algorithmic work of a batch (for the roofline report)
# ----------------------------------------------------------------------------
def work_of(shape: LayerShape, b: Batch) -> Dict[str, float]:
    """FLOPs and HBM bytes one step must do: weights once, x in and y out, KV
    append, every referenced KV page once per prefix node (and, for comparison,
    once per sequence), causal half of prefill attention."""
    T = b.n_rows
    hq, dh = shape.n_q_heads, shape.head_dim
    q_len = b.q_len().astype(np.int64)
    kv = b.kv_len.astype(np.int64)
    c = kv - q_len
    gemm_flops = 2.0 * T * shape.matrix_params
    pre = slice(0, b.n_prefill)
    dec = slice(b.n_prefill, b.n_seq)
    pre_attn = 4.0 * hq * dh * float(np.sum(q_len[pre] * c[pre] + q_len[pre] * (q_len[pre] + 1) // 2))
    dec_attn = 4.0 * hq * dh * float(np.sum(kv[dec]))
    kappa = shape.kv_bytes_per_token
    n_tab = np.diff(b.page_start).astype(np.int64)
    # tokens read from cache: every token of every sequence's context, whole pages for shared parts
    expanded_tokens = float(np.sum(kv))
    shared_pages_per_seq = np.zeros(b.n_seq, dtype=np.int64)
    node_np = np.diff(b.node_page_start).astype(np.int64)
    path_pages = np.zeros(b.n_nodes, dtype=np.int64)
    for i in range(b.n_nodes):
        p = int(b.node_parent[i])
        path_pages[i] = node_np[i] + (path_pages[p] if p >= 0 else 0)
    for s in range(b.n_seq):
        l = int(b.seq_leaf_node[s])
        if l >= 0:
            shared_pages_per_seq[s] = path_pages[l]
    live_nodes = node_np[b.node_seq_count > 0] if b.n_nodes else node_np
    once_tokens = float(np.sum(kv - shared_pages_per_seq * b.page_size) + np.sum(live_nodes) * b.page_size)
    w_bytes = 2.0 * shape.matrix_params + 2.0 * 2 * shape.d_model
    act_bytes = 2.0 * 2 * T * shape.d_model
    append_bytes = float(T * kappa)
    bytes_once = w_bytes + act_bytes + append_bytes + once_tokens * kappa
    bytes_exp = w_bytes + act_bytes + append_bytes + expanded_tokens * kappa
    return dict(rows=T, gemm_flops=gemm_flops, prefill_attn_flops=pre_attn, decode_attn_flops=dec_attn,
                flops=gemm_flops + pre_attn + dec_attn, weight_bytes=w_bytes,
                kv_tokens_once=once_tokens, kv_tokens_expanded=expanded_tokens,
                bytes_once=bytes_once, bytes_expanded=bytes_exp, table_pages=float(np.sum(n_tab)))


# ----------------------------------------------------------------------------
# a request pool for the multi-step driver
# ----------------------------------------------------------------------------
@dataclass
class PoolRequest:
    tokens: Sequence[int]
    d_est: int      # the estimate that ordering, admission and reservation see
    d_true: int     # the length after which the request ends


def synthetic_pool(seed: int, n_groups: int = 24, per_group: int = 12, n_fresh: int = 96, est_noise: float = 0.25,
                   templates: str = "by_kind") -> List[PoolRequest]:
    """A pool with the structure of the paper's mixed workloads (Section 6.1): groups sharing a
    long system prompt whose members generate short outputs (compute-intensive, benchmark-like),
    groups with medium and with long outputs (memory-intensive), and unrelated prompt-heavy
    requests.  Each kind comes from its own dataset, whose prompts start with the same template
    token, so a prefix-DFS order serves one dataset after the other, as it would a concatenation
    of traces.  templates="by_kind" numbers the template tokens so that the DFS order meets the
    compute-intensive datasets first and the long-output one last (the case Section 3.1 describes
    as hurting it); templates="shuffled" numbers them at random (a neutral order for that
    baseline).  Output-length estimates are the true lengths with multiplicative noise."""
    assert templates in ("by_kind", "shuffled")
    rng = np.random.default_rng(seed)
    tpl = [0, 1, 2, 3] if templates == "by_kind" else [int(t) for t in np.random.default_rng([seed, 7]).permutation(4)]
    out: List[PoolRequest] = []
    for g in range(n_groups):
        kind = g % 3
        prefix = [tpl[kind + 1]] + [int(t) for t in rng.integers(4, 128000, int(rng.integers(256, 1536)))]
        for _ in range(per_group):
            own = [int(t) for t in rng.integers(4, 128000, int(rng.integers(16, 256)))]
            d = int(rng.integers(8, 48)) if kind == 0 else int(rng.integers(128, 512)) if kind == 1 else int(rng.integers(768, 2048))
            out.append(PoolRequest(prefix + own, 0, d))
    for _ in range(n_fresh):
        toks = [tpl[0]] + [int(t) for t in rng.integers(4, 128000, int(rng.integers(512, 3072)))]
        out.append(PoolRequest(toks, 0, int(rng.integers(4, 64))))
    for r in out:
        r.d_est = max(1, int(round(r.d_true * float(np.exp(est_noise * rng.standard_normal())))))
    perm = rng.permutation(len(out))
    return [out[i] for i in perm]


def baseline_order(reqs: Sequence[PoolRequest], policy: str, seed: int = 0) -> List[int]:
    """Request orders that the resource-aware order is compared with (Section 6.3): "dfs" = prompts in
    lexicographic order, i.e. the DFS order of the plain prefix tree (best sharing); "random"."""
    if policy == "dfs":
        return sorted(range(len(reqs)), key=lambda i: (list(reqs[i].tokens), i))
    if policy == "random":
        return [int(i) for i in np.random.default_rng(seed).permutation(len(reqs))]
    raise ValueError("unknown baseline order " + policy)


CONFIGS = {
    "tiny": (TINY, batch_tiny),
    "decode_8b": (LLAMA3_8B, batch_decode_only),
    "prefill_8b": (LLAMA3_8B, batch_prefill_only),
    "blended_8b": (LLAMA3_8B, batch_blended_8b),
    "blended_70b": (LLAMA3_70B, batch_blended_70b),
}
