"""CPU oracle of the host-side batch builder (resource-aware prefix tree, layer-wise
sort, dual scan).  TEST INFRASTRUCTURE ONLY: the product path never imports this.

This part of BlendServe is a heuristic, so the oracle is the algorithm itself,
step by step in the paper's order and notation, written in plain Python with
exact integer / rational arithmetic where a decision depends on a comparison.

  1. Prefix tree (Section 5.1): a compressed trie over the prompt token ids; every
     request is a leaf, every internal node is a maximal prompt segment shared by
     all requests below it.
  2. Compute density of a node (Section 5.1, rho(R) = (1-s) T_comp / T_mem, with the
     request model of Section 4.1 after its p^2 term is dropped):
        (1-s) T_comp = 2 P_model * A(R) / compute,
            A(R) = distinct prompt tokens of the subtree, counting the path from the
                   root to R once, + sum of output lengths d_i
        T_mem       = kappa * B(R) / (2 bandwidth),   B(R) = sum_i (2 p_i d_i + d_i^2)
     (kappa = bytes of K and V per token over all layers, "H_kv * L * 4"; the sum of
     (p + i) for i = 1..d is p d + d^2/2 as in the paper, i.e. B/2).
     Nodes are compared exactly through A1 * B2 versus A2 * B1; B = 0 is +infinity.
  3. Layer-wise sort (Algorithm 1): at every internal node the children are ordered by
     density, compute-intensive first; ties go to the subtree holding the smaller
     request index.  Only siblings move, so the trie itself is unchanged.
  4. Nodes are numbered in DFS pre-order of the sorted tree; the leaves from left to
     right are the compute-to-memory request order.
  5. Dual scan (Algorithm 3; Section 5.3): with R_L / R_R the leftmost / rightmost
     subtree under the (first branching) root,
        M_L = M (rho(rt) - rho(R_R)) / (rho(R_L) - rho(R_R)),  M_R = M - M_L,
        N_X = M_X / ((p_X + d_X / 2) kappa),   C_X = N_X p_X / d_X,
     p_X, d_X the mean prompt and output length of side X.  Readings where the paper
     is silent: equal densities give M_L = M; M_L is clamped to [0, M]; N and C are
     floored, N to at least one request per side; a side without decode work
     (d_X = 0) gets an unlimited prefill budget.
     One step then admits, scanning the leaves inwards from both ends, up to N_X
     decoding requests and up to C_X prefill tokens per side (the last admitted
     prompt may be cut: chunked prefill), and emits the batch descriptor: prefill
     segments first, decode sequences in leaf order, prefix nodes = trie nodes with
     at least two admitted decode members and at least one whole KV page, each
     node's pages allocated once.

  6. Conditional node splitting (Section 5.2, Algorithm 2, and the stopping conditions
     of Section 5.4).  The printed pseudo-code and the prose disagree (the listing
     splits when prefix length x children exceeds t and divides t among children; the
     text relocates a leaf when its recomputation cost is BELOW t); this follows the
     text and the convergence argument.  One round:
       a. the leaf densities rho(r) = (p + d) / (2 p d + d^2), left to right, are
          examined; if they are non-increasing the search stops (C1);
       b. outliers, first kind (the figure's case: a request of low density among
          compute-intensive ones drags the density of every subtree that holds it,
          since rho of a node is sum A / sum B): a leaf l below a non-root node X such
          that X without l would change places with the sibling Q next to it, while l
          itself belongs on the far side of all of Q (X jumps left over Q and l is
          less dense than every leaf of Q, or the mirror image);
          second kind, only when there is none of the first: the leaves outside a
          longest non-increasing subsequence (patience procedure of
          `longest_non_increasing`, which fixes the choice among equally long ones); a
          leaf that is already a direct child of the root cannot move, so where such a
          leaf is the outlier of an adjacent violation rho(i) < rho(i+1), its
          neighbour is taken instead;
       c. a candidate's cost is its shared prefix length (the tokens recomputed once
          it no longer shares them); candidates with cost <= t are taken cheapest
          first (ties: smaller request index) while the total stays within the
          budget; none taken = stop (C2);
       d. every taken leaf is cut from its parent and re-inserted as a direct child of
          the root with its whole prompt as its own segment; the trie of the others is
          rebuilt (a parent left with one child merges with it), densities are
          recomputed and Algorithm 1 runs again.
     Every leaf is split at most once, so there are at most N_leaf rounds.

  7. Memory model with prefix pages read once (an extension: Section 3.3 charges the
     cached prefix of every request at full bytes because a prefix-cache hit saves no
     bandwidth; with the intra-batch prefix sharing of Appendix A.2 the pages of a shared
     segment are read once per step for all requests below it).  `mem_model="shared"`
     replaces B(R) by the loaded-token count of the subtree when all its requests decode
     together, each segment charged once per step while any request below it still
     decodes:
        S(leaf) = 2 own d + d^2,           D(leaf) = d,
        S(N)    = 2 len(N) D(N) + sum_c S(c),   D(N) = max_c D(c),
        B(R)    = S(R) + 2 start(R) D(R)        (the path above R, shared by all of R),
     which equals the paper's B wherever nothing is shared.  A is unchanged.  Node
     splitting (step 6) reasons with sums over leaves and is defined for the paper's
     model only.  The other attention variants of Section 7 (MHA, MQA, GQA, MLA) enter
     through kappa alone: `kv_bytes_per_token`.

Pins (tests/test_oracle_builder.py): the memory-partition example printed with
Figure 6; the batch-density = request-density identity of Section 4.2; linearity of
the memory model in loaded tokens (the ratios of Table 1); brute-force shared-prefix
lengths, distinct-token counts and sibling order on small random pools; the
invariants that sorting keeps every parent's child set and that every node's
requests are contiguous in leaf order.  Admission (`next_batch`): a pool of six
requests whose M_L, M_R, N_X, C_X are worked out by hand from Algorithm 3's formulas
in exact fractions, with the requests and chunk lengths that each scanner then admits
written out, also under prefill and decode caps.  Descriptor (`emit`): the page tables,
node pages, member runs and leaf nodes of that step and of a two-level prefix tree
written out by hand.  Absolute densities of the paper's traces need its datasets:
parity unpinned for those.  Node splitting: its bounds and invariants (no round
without a split, at most N_leaf splits, t = 0 changes nothing, unlimited t ends in a
non-increasing leaf order, sharing lost = the sum of the costs, the worked example of
Figure 3 where the low-density request moves to the right end) and the stopping
conditions of Section 5.4 by enumeration on pools of at most six leaves: the search
ends with non-increasing leaf densities (C1) or with no affordable split left (C2)
among the leaves that lie in no longest non-increasing subsequence at all; which
leaves are taken as outliers where several choices are equally good is this file's
reading: parity unpinned for that choice.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction
from typing import List, Optional, Sequence, Tuple

import numpy as np


def kv_bytes_per_token(variant: str, n_layers: int, n_heads: int, head_dim: int, n_kv_heads: int = 0,
                       latent_dim: int = 0, rope_dim: int = 0, elem_bytes: int = 2) -> int:
    """kappa of Section 4.1 ("H_kv * L * 2 * 2": keys and values of every KV head, every
    layer, 2 bytes each) for the attention variants named in Section 7.  MHA keeps one KV
    head per query head, MQA one in all, GQA n_kv_heads; MLA caches one compressed latent
    of latent_dim plus a shared rotary key of rope_dim per token and layer instead of
    per-head keys and values."""
    if variant == "mha":
        per_layer = 2 * n_heads * head_dim
    elif variant == "mqa":
        per_layer = 2 * head_dim
    elif variant == "gqa":
        if n_kv_heads <= 0 or n_heads % n_kv_heads:
            raise ValueError("gqa needs n_kv_heads dividing n_heads")
        per_layer = 2 * n_kv_heads * head_dim
    elif variant == "mla":
        if latent_dim <= 0:
            raise ValueError("mla needs latent_dim")
        per_layer = latent_dim + rope_dim
    else:
        raise ValueError("unknown attention variant " + variant)
    return per_layer * n_layers * elem_bytes


@dataclass
class CostModel:
    p_model: int          # model parameters
    kv_bytes: int         # kappa: bytes of K and V per token over all layers
    compute: float        # FLOP/s
    bandwidth: float      # bytes/s
    mem_bytes: int        # M: KV-cache capacity in bytes
    page_size: int = 16
    mem_model: str = "expanded"   # "expanded": Section 4.1's Mem(r) summed; "shared": step 7 above


@dataclass
class Request:
    tokens: Sequence[int]
    d_est: int
    n_cached: int = 0     # tokens whose KV is cached; >= len(tokens) means the request is decoding


@dataclass
class TNode:
    start: int                      # token depth where the node's segment starts
    end: int                        # token depth where it ends (exclusive)
    parent: int
    children: List[int] = field(default_factory=list)
    req: int = -1                   # request index for a leaf, else -1
    A: int = 0
    B: int = 0
    n_req: int = 0
    sum_p: int = 0
    sum_d: int = 0
    min_req: int = 0
    S: int = 0                      # "shared" memory model: loaded tokens (x2) at or below the node's segment
    max_d: int = 0                  # longest output below the node
    lo: Tuple[int, int] = (0, 1)    # (A, B) of the least / most compute-intensive leaf below
    hi: Tuple[int, int] = (0, 1)


def density_fraction(A: int, B: int) -> Optional[Fraction]:
    """A / B as an exact fraction (the hardware constants cancel in comparisons); None = +inf."""
    return None if B == 0 else Fraction(A, B)


def denser(a: Tuple[int, int], b: Tuple[int, int]) -> int:
    """+1 if node a = (A, B) is strictly more compute-intensive than b, -1 if less, 0 if equal."""
    (A1, B1), (A2, B2) = a, b
    if B1 == 0 and B2 == 0:
        return 0
    if B1 == 0:
        return 1
    if B2 == 0:
        return -1
    l, r = A1 * B2, A2 * B1
    return (l > r) - (l < r)


def rho_value(cm: CostModel, A: int, B: int) -> float:
    """rho(R) = [2 P_model A / compute] / [kappa B / (2 bandwidth)] in double precision,
    operations in exactly this order (the C++ builder repeats them)."""
    if B == 0:
        return float("inf")
    t_comp = (2.0 * float(cm.p_model)) * float(A) / cm.compute
    t_mem = (float(cm.kv_bytes) * float(B)) / (2.0 * cm.bandwidth)
    return t_comp / t_mem


def memory_partition(rho_rt: float, rho_l: float, rho_r: float, M: float) -> Tuple[float, float]:
    """Algorithm 3, step 1.  M_L + M_R = M and M_L rho_L + M_R rho_R = M rho_rt."""
    if rho_l == rho_r or rho_l == float("inf"):
        m_l = M if rho_l == rho_r else (0.0 if rho_rt != float("inf") else M)
    else:
        m_l = M * ((rho_rt - rho_r) / (rho_l - rho_r))
    m_l = min(max(m_l, 0.0), M)
    return m_l, M - m_l


def longest_non_increasing(keys: Sequence[Tuple[int, int]]) -> List[int]:
    """Indices of a longest non-increasing subsequence of densities (A, B), by patience:
    pile k holds the index of the densest last element of any non-increasing subsequence of
    length k + 1 seen so far; a new element goes to the first pile whose last element is
    strictly less dense than it (else it opens a new pile) and remembers the top of the
    pile before; the answer is read back from the top of the last pile."""
    tails: List[int] = []
    pred = [-1] * len(keys)
    for i, k in enumerate(keys):
        lo, hi = 0, len(tails)
        while lo < hi:                              # first pile whose tail is strictly less dense than k
            mid = (lo + hi) // 2
            if denser(k, keys[tails[mid]]) > 0:
                hi = mid
            else:
                lo = mid + 1
        pred[i] = tails[lo - 1] if lo > 0 else -1
        if lo == len(tails):
            tails.append(i)
        else:
            tails[lo] = i
    out: List[int] = []
    i = tails[-1] if tails else -1
    while i >= 0:
        out.append(i)
        i = pred[i]
    out.reverse()
    return out


class BuilderOracle:
    def __init__(self, cm: CostModel, requests: Sequence[Request]):
        self.cm = cm
        self.reqs = list(requests)
        self.nodes: List[TNode] = []
        self.detached: set = set()             # requests re-inserted under the root by node splitting
        self._rebuild()

    def _rebuild(self):
        self.nodes = []
        self._build_trie()
        for r in sorted(self.detached):
            leaf = len(self.nodes)
            self.nodes.append(TNode(0, len(self.reqs[r].tokens), 0, req=r))
            self.nodes[0].children.append(leaf)
        self._annotate(0)
        self._layer_sort(0)
        self._number()

    # -- step 6: conditional node splitting ----------------------------------------------
    def leaf_keys(self) -> List[Tuple[int, int]]:
        leaf_of = {nd.req: nd for nd in self.nodes if nd.req >= 0}
        return [(leaf_of[r].A, leaf_of[r].B) for r in self.leaf_order]

    def split(self, t: int, budget: int = -1):
        """Relocate outlier leaves whose shared prefix is at most t tokens, spending at most
        `budget` recomputed tokens in total (< 0: no limit)."""
        if self.cm.mem_model != "expanded":
            raise ValueError("node splitting is defined for the paper's memory model only")
        spent = rounds = n_split = 0
        while True:
            keys = self.leaf_keys()
            n = len(keys)
            kept = set(longest_non_increasing(keys))
            if len(kept) == n:
                break                                              # C1
            leaf_of = {nd.req: nd for nd in self.nodes if nd.req >= 0}
            movable = [leaf_of[r].parent != 0 for r in self.leaf_order]
            cand = set()
            for i, r in enumerate(self.leaf_order):                # first kind
                lf = leaf_of[r]
                if not movable[i]:
                    continue
                gone = (lf.A - lf.start, lf.B)                      # what every ancestor loses with the leaf
                x = lf.parent
                while x != 0 and i not in cand:
                    X = self.nodes[x]
                    sib = self.nodes[X.parent].children
                    j = sib.index(x)
                    rest = (X.A - gone[0], X.B - gone[1])
                    if j > 0:
                        Q = self.nodes[sib[j - 1]]
                        if denser(rest, (Q.A, Q.B)) > 0 and denser((lf.A, lf.B), Q.lo) < 0:
                            cand.add(i)
                    if j + 1 < len(sib):
                        Q = self.nodes[sib[j + 1]]
                        if denser(rest, (Q.A, Q.B)) < 0 and denser((lf.A, lf.B), Q.hi) > 0:
                            cand.add(i)
                    x = X.parent
            if not cand:                                           # second kind
                cand = {i for i in range(n) if i not in kept and movable[i]}
                for i in range(n - 1):
                    if denser(keys[i], keys[i + 1]) < 0 and i not in cand and (i + 1) not in cand:
                        # the outlier of this violation sits under the root already: move its neighbour
                        if i not in kept and movable[i + 1]:
                            cand.add(i + 1)
                        elif (i + 1) not in kept and movable[i]:
                            cand.add(i)
            todo = sorted((leaf_of[self.leaf_order[i]].start, self.leaf_order[i]) for i in cand
                          if leaf_of[self.leaf_order[i]].start <= t)
            took = 0
            for cost, r in todo:
                if budget >= 0 and spent + cost > budget:
                    break
                self.detached.add(r)
                spent += cost
                took += 1
            if took == 0:
                break                                              # C2
            n_split += took
            rounds += 1
            self._rebuild()
        keys = self.leaf_keys()
        monotone = all(denser(keys[i], keys[i + 1]) >= 0 for i in range(len(keys) - 1))
        return dict(n_split=n_split, rounds=rounds, recompute_tokens=spent, monotone=monotone)

    # -- step 1: compressed trie through sorted prompts and longest common prefixes --------
    def _build_trie(self):
        reqs = self.reqs
        order = sorted((i for i in range(len(reqs)) if i not in self.detached), key=lambda i: (list(reqs[i].tokens), i))
        self.nodes = [TNode(0, 0, -1)]          # root: empty segment
        stack = [0]                             # path of internal nodes, root first
        prev_tokens: Optional[Sequence[int]] = None
        prev_leaf = -1
        for i in order:
            tok = list(reqs[i].tokens)
            lcp = 0
            if prev_tokens is not None:
                n = min(len(tok), len(prev_tokens))
                while lcp < n and tok[lcp] == prev_tokens[lcp]:
                    lcp += 1
                # climb to the deepest internal node that ends at or above lcp
                while self.nodes[stack[-1]].end > lcp:
                    stack.pop()
                top = stack[-1]
                if self.nodes[top].end < lcp:
                    # split below `top`: the previous path continues past lcp, so a new internal
                    # node [top.end, lcp) adopts the child of `top` that holds the previous leaf
                    child = self.nodes[top].children[-1]
                    mid = len(self.nodes)
                    self.nodes.append(TNode(self.nodes[top].end, lcp, top))
                    self.nodes[top].children[-1] = mid
                    self.nodes[mid].children.append(child)
                    self.nodes[child].parent = mid
                    self.nodes[child].start = lcp
                    stack.append(mid)
            top = stack[-1]
            leaf = len(self.nodes)
            self.nodes.append(TNode(self.nodes[top].end, len(tok), top, req=i))
            self.nodes[top].children.append(leaf)
            prev_tokens, prev_leaf = tok, leaf

    # -- step 2: bottom-up A, B and bookkeeping ------------------------------------------
    def _annotate(self, n: int):
        nd = self.nodes[n]
        if nd.req >= 0:
            r = self.reqs[nd.req]
            p, d = len(r.tokens), int(r.d_est)
            nd.n_req, nd.sum_p, nd.sum_d, nd.min_req = 1, p, d, nd.req
            own = nd.end - nd.start
            nd.B = 2 * p * d + d * d
            nd.S, nd.max_d = 2 * own * d + d * d, d
            below = own + d                       # distinct tokens strictly below the node's start
            nd.lo = nd.hi = (nd.start + below, nd.B)
        else:
            below = nd.end - nd.start
            nd.n_req = nd.sum_p = nd.sum_d = nd.B = nd.S = nd.max_d = 0
            nd.min_req = 1 << 62
            for k, c in enumerate(nd.children):
                self._annotate(c)
                ch = self.nodes[c]
                nd.lo = ch.lo if k == 0 or denser(ch.lo, nd.lo) < 0 else nd.lo
                nd.hi = ch.hi if k == 0 or denser(ch.hi, nd.hi) > 0 else nd.hi
                nd.n_req += ch.n_req
                nd.sum_p += ch.sum_p
                nd.sum_d += ch.sum_d
                nd.B += ch.B
                nd.S += ch.S
                nd.max_d = max(nd.max_d, ch.max_d)
                nd.min_req = min(nd.min_req, ch.min_req)
                below += ch.A - ch.start          # the child's A counts its root path once: remove it
            nd.S += 2 * (nd.end - nd.start) * nd.max_d
            if self.cm.mem_model == "shared":
                nd.B = nd.S + 2 * nd.start * nd.max_d
        nd.A = nd.start + below                   # the path root -> node counted once
        return nd

    # -- step 3: Algorithm 1 -------------------------------------------------------------
    def _layer_sort(self, n: int):
        nd = self.nodes[n]
        if nd.req >= 0:
            return
        import functools

        def cmp(a: int, b: int) -> int:
            x, y = self.nodes[a], self.nodes[b]
            c = denser((x.A, x.B), (y.A, y.B))
            if c:
                return -c                          # denser first
            return (x.min_req > y.min_req) - (x.min_req < y.min_req)
        nd.children.sort(key=functools.cmp_to_key(cmp))
        for c in nd.children:
            self._layer_sort(c)

    # -- step 4: DFS numbering -----------------------------------------------------------
    def _number(self):
        self.dfs: List[int] = []               # node ids in pre-order
        self.leaf_order: List[int] = []        # request indices left to right
        self.first_leaf = {}
        self.leaf_count = {}
        stack = [0]
        # iterative pre-order
        def visit(n):
            self.dfs.append(n)
            nd = self.nodes[n]
            self.first_leaf[n] = len(self.leaf_order)
            if nd.req >= 0:
                self.leaf_order.append(nd.req)
            for c in nd.children:
                visit(c)
            self.leaf_count[n] = len(self.leaf_order) - self.first_leaf[n]
        import sys
        sys.setrecursionlimit(max(10000, sys.getrecursionlimit()))
        visit(0)
        self.dfs_index = {n: i for i, n in enumerate(self.dfs)}

    def tree_arrays(self):
        """The sorted tree as arrays in DFS pre-order (what the C++ builder must reproduce)."""
        n = len(self.dfs)
        parent = np.full(n, -1, dtype=np.int32)
        start = np.zeros(n, dtype=np.int32)
        end = np.zeros(n, dtype=np.int32)
        req = np.full(n, -1, dtype=np.int32)
        first = np.zeros(n, dtype=np.int32)
        count = np.zeros(n, dtype=np.int32)
        A = np.zeros(n, dtype=np.int64)
        B = np.zeros(n, dtype=np.int64)
        for i, nid in enumerate(self.dfs):
            nd = self.nodes[nid]
            parent[i] = self.dfs_index[nd.parent] if nd.parent >= 0 else -1
            start[i], end[i], req[i] = nd.start, nd.end, nd.req
            first[i], count[i] = self.first_leaf[nid], self.leaf_count[nid]
            A[i], B[i] = nd.A, nd.B
        return dict(parent=parent, start=start, end=end, req=req, first_leaf=first, leaf_count=count, A=A, B=B,
                    leaf_order=np.asarray(self.leaf_order, dtype=np.int32))

    # -- step 5: Algorithm 3 and one step's admission ------------------------------------
    def scan_sides(self):
        """(root-like node, R_L, R_R): descend single-child chains to the first branching node."""
        n = 0
        while self.nodes[n].req < 0 and len(self.nodes[n].children) == 1:
            n = self.nodes[n].children[0]
        nd = self.nodes[n]
        if nd.req >= 0 or len(nd.children) < 2:
            return n, n, n
        return n, nd.children[0], nd.children[-1]

    def budgets(self):
        cm = self.cm
        rt, L, R = self.scan_sides()
        nrt, nl, nr = self.nodes[rt], self.nodes[L], self.nodes[R]
        rho_rt, rho_l, rho_r = (rho_value(cm, x.A, x.B) for x in (nrt, nl, nr))
        m_l, m_r = memory_partition(rho_rt, rho_l, rho_r, float(cm.mem_bytes))
        out = dict(rho_rt=rho_rt, rho_l=rho_l, rho_r=rho_r, m_l=m_l, m_r=m_r)
        for tag, nd, m in (("l", nl, m_l), ("r", nr, m_r)):
            p_bar = float(nd.sum_p) / float(nd.n_req)
            d_bar = float(nd.sum_d) / float(nd.n_req)
            n_dec = max(1, int(np.floor(m / ((p_bar + d_bar / 2.0) * float(cm.kv_bytes)))))   # a side is never starved
            c_pre = -1 if d_bar == 0.0 else int(np.floor(float(n_dec) * p_bar / d_bar))
            out["n_" + tag], out["c_" + tag] = n_dec, c_pre
        return out

    def next_batch(self, prefill_budget: int = 0, decode_budget: int = 0):
        """One step's batch.  Budgets <= 0 mean "no extra cap"."""
        cm, ps = self.cm, self.cm.page_size
        b = self.budgets()
        n_l, n_r, c_l, c_r = b["n_l"], b["n_r"], b["c_l"], b["c_r"]
        INF = 1 << 60
        c_l = INF if c_l < 0 else c_l
        c_r = INF if c_r < 0 else c_r
        if prefill_budget > 0 and c_l + c_r > prefill_budget:
            if c_l >= INF and c_r >= INF:
                c_l = prefill_budget // 2
            elif c_l >= INF:
                c_l = max(0, prefill_budget - c_r)
            elif c_r >= INF:
                c_l = min(c_l, prefill_budget)
            else:
                c_l = c_l * prefill_budget // (c_l + c_r)
            c_r = prefill_budget - c_l
        if decode_budget > 0 and n_l + n_r > decode_budget:
            n_l = n_l * decode_budget // (n_l + n_r)
            n_r = decode_budget - n_l
        order = self.leaf_order
        taken = {}
        pre: List[Tuple[int, int]] = []        # (request, chunk rows) in admission order
        dec_l: List[int] = []
        dec_r: List[int] = []

        def admit(ri: int, side: str) -> bool:
            nonlocal n_l, n_r, c_l, c_r
            r = self.reqs[ri]
            p = len(r.tokens)
            if r.n_cached >= p:                  # decoding
                if side == "l" and n_l > 0:
                    n_l -= 1; dec_l.append(ri); return True
                if side == "r" and n_r > 0:
                    n_r -= 1; dec_r.append(ri); return True
                return False
            left = c_l if side == "l" else c_r
            if left <= 0:
                return False
            chunk = min(p - r.n_cached, left)
            pre.append((ri, chunk))
            if side == "l":
                c_l -= chunk
            else:
                c_r -= chunk
            return True

        i, j = 0, len(order) - 1
        # alternate the two scanners; a scanner stops for good at its first refusal
        go_l = go_r = True
        while i <= j and (go_l or go_r):
            if go_l and i <= j:
                if admit(order[i], "l"):
                    i += 1
                else:
                    go_l = False
            if go_r and i <= j:
                if admit(order[j], "r"):
                    j -= 1
                else:
                    go_r = False
        dec = dec_l + dec_r
        b.update(n_prefill=len(pre), n_decode=len(dec))
        desc = self.emit([(ri, self.reqs[ri].n_cached, chunk) for ri, chunk in pre],
                         [(ri, self.reqs[ri].n_cached) for ri in dec])
        return b, desc

    def emit(self, pre: Sequence[Tuple[int, int, int]], dec: Sequence[Tuple[int, int]]):
        """The batch descriptor of an explicit step: prefill segments (request, tokens already
        cached, rows this step) in the order given, then decode sequences (request, tokens cached
        before this step) in leaf order.  Prefix nodes = trie nodes with at least two of the decode
        sequences below them and at least one whole page of their own; pages are numbered afresh:
        node pages first (DFS order), then every sequence's private pages."""
        ps = self.cm.page_size
        order = self.leaf_order
        pos_in_order = {ri: k for k, ri in enumerate(order)}
        ctx_of = {ri: c for ri, c in dec}
        cached_of = {ri: c for ri, c, _ in pre}
        pre = [(ri, chunk) for ri, _, chunk in pre]
        dec = sorted((ri for ri, _ in dec), key=lambda ri: pos_in_order[ri])
        # ---- descriptor ----------------------------------------------------------------
        # prefix nodes: trie nodes (in DFS order) with >= 2 admitted decode members and >= 1 whole page
        dec_pos = {ri: k for k, ri in enumerate(dec)}
        leaf_node_of_req = {self.nodes[n].req: n for n in self.dfs if self.nodes[n].req >= 0}
        members = {}
        for ri in dec:
            n = self.nodes[leaf_node_of_req[ri]].parent
            while n >= 0:
                members.setdefault(n, []).append(dec_pos[ri])
                n = self.nodes[n].parent
        kept = []                                  # (trie node, page_lo, page_hi)
        node_id = {}
        cover = {}                                 # trie node -> pages covered by kept ancestors incl. itself
        node_parent, node_first, node_count, node_pages = [], [], [], []
        for n in self.dfs:
            nd = self.nodes[n]
            if nd.req >= 0:
                continue
            par = nd.parent
            above = cover.get(par, 0) if par >= 0 else 0
            hi = nd.end // ps
            m = members.get(n, [])
            if len(m) >= 2 and hi > above:
                anc = par
                while anc >= 0 and anc not in node_id:
                    anc = self.nodes[anc].parent
                node_id[n] = len(node_parent)
                node_parent.append(node_id[anc] if anc >= 0 else -1)
                node_first.append(len(pre) + min(m))
                node_count.append(len(m))
                node_pages.append((above, hi))
                cover[n] = hi
            else:
                cover[n] = above
        next_page = 0
        node_page_start = [0]
        node_page_ids: List[int] = []
        for lo, hi in node_pages:
            node_page_ids.extend(range(next_page, next_page + hi - lo))
            next_page += hi - lo
            node_page_start.append(len(node_page_ids))
        row_start, kv_len, page_start, page_ids, seq_leaf, seq_req = [0], [], [0], [], [], []
        for ri, chunk in pre:
            r = self.reqs[ri]
            kv = cached_of[ri] + chunk
            npg = -(-kv // ps)
            page_ids.extend(range(next_page, next_page + npg))
            next_page += npg
            row_start.append(row_start[-1] + chunk)
            kv_len.append(kv); page_start.append(len(page_ids)); seq_leaf.append(-1); seq_req.append(ri)
        for ri in dec:
            r = self.reqs[ri]
            kv = ctx_of[ri] + 1
            # deepest kept node on the request's path
            n = self.nodes[leaf_node_of_req[ri]].parent
            while n >= 0 and n not in node_id:
                n = self.nodes[n].parent
            leaf = node_id[n] if n >= 0 else -1
            path = []
            k = leaf
            while k >= 0:
                path.append(k)
                k = node_parent[k]
            shared = 0
            for k in reversed(path):
                page_ids.extend(node_page_ids[node_page_start[k]:node_page_start[k + 1]])
                shared += node_page_start[k + 1] - node_page_start[k]
            npg = -(-kv // ps)
            page_ids.extend(range(next_page, next_page + npg - shared))
            next_page += npg - shared
            row_start.append(row_start[-1] + 1)
            kv_len.append(kv); page_start.append(len(page_ids)); seq_leaf.append(leaf); seq_req.append(ri)
        i32 = lambda a: np.asarray(a, dtype=np.int32)
        desc = dict(n_seq=len(pre) + len(dec), n_prefill=len(pre), n_rows=row_start[-1],
                    row_start=i32(row_start), kv_len=i32(kv_len), page_start=i32(page_start), page_ids=i32(page_ids),
                    n_nodes=len(node_parent), node_parent=i32(node_parent), node_page_start=i32(node_page_start),
                    node_page_ids=i32(node_page_ids), node_seq_first=i32(node_first), node_seq_count=i32(node_count),
                    seq_leaf_node=i32(seq_leaf), seq_request=i32(seq_req), n_pages=next_page)
        return desc
