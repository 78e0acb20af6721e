"""CPU oracle of the multi-step driver: a pool of requests served to completion, one batch
descriptor per step, with KV pages that keep their physical number from the step that writes
them to the step that frees them.  TEST INFRASTRUCTURE ONLY: the product path never imports this.

What it follows.  BlendServe re-forms the runtime batch every iteration (Section 3.2, Appendix
A.2 "batch scheduler"): every decoding request contributes one row, the rest of the token
budget goes to prefill chunks (Section 2.2, chunked prefill), and new requests are admitted from
the two ends of the sorted leaf order, one scanner per end, the KV memory split between the two
by Algorithm 3 (Section 5.3).  Output lengths are estimates; Section 5.4 names the adaptation:
a request that ends early frees its memory at once, one that runs past its estimate keeps
growing, and a severely underestimated one is moved from the compute-intensive partition to the
memory-intensive one.  Prefix sharing is kept at run time by a prefix tree (Appendix A.2): a
shared prompt segment is computed once, by the first resident request that needs it, and its
KV pages are referenced by every request below it.

The paper gives these mechanisms in words; the steps below are this build's reading, stated so
that two implementations agree bit for bit.  Plain Python, integers only after the initial
partition (two doubles, evaluated in the order written).

State
  order          leaf order of the sorted tree (compute-intensive first), or a given order
  lo, hi         next candidates of the left and the right scanner (a given order: left only)
  cap[2]         memory of each side in tokens: cap[0] = floor(M * (M_L / (M_L + M_R))), M in tokens
  pre_num/den    share of a step's prefill budget that the left side may take: C_L / (C_L + C_R)
                 of Algorithm 3 (1/2 where a side's C is unlimited or both are zero)
  p_side[2]      mean prompt length of each side's subtree, rounded up (the p of Algorithm 3)
  per request    side, cached (prompt tokens whose KV exists), generated, reserved (tokens
                 charged for it alone), private pages
  per segment    (internal trie node with a non-empty segment) ref = resident requests below,
                 done = tokens of the segment computed, owner = the request computing it,
                 side = the partition that was charged for it, pages

Pages.  Sharing is page-granular.  Node n shares the logical pages [lo_n, hi_n) of every request
below it, lo_n = hi_parent (0 at the top), hi_n = end_n // 16, or (end_n - 1) // 16 where some
request's prompt ends exactly at end_n (its last prompt row must have a private slot to be
written to); hi_n is never below lo_n.  Every other logical page of a request is private.  A
physical page is taken from the free pool (smallest number first) when a step first writes a
token into it and returned when its request finishes (private) or when the last resident
request below its node leaves (shared).

One step
  1. Every live request whose prompt is cached contributes a decode row at position
     p + generated - 1.  The rest of the token budget B is for prefill:
     left share = floor(B * pre_num / pre_den), right share = B - left share, except that
     neither scanner is starved (Algorithm 3 keeps both partitions filled; the reading "at
     least one request per side" applied to a step): each side's share is at least
     min(p_side, floor(B / 2)), the chunk that admits one average request of that side.
  2. Requests admitted earlier whose prompt is not yet cached continue, in admission order, each
     with a chunk of min(tokens left, its side's share); those whose side has nothing left wait.
  3. First pass: the scanners take turns, left first.  A scanner admits its next request if
       a. no segment on its path is still being computed by another request (else it waits:
          the scanner stops for this step), and
       b. used[side] + need <= cap[side], need = its own segment + its estimated output + the
          segments on its path that no resident request holds; a request that would be the
          only live one is admitted regardless (nothing would ever free memory for it).
     An admitted request starts behind the whole pages of the complete segments at the head of
     its path (cached = 16 * hi of the deepest such node; at most p - 1, so that one row is left)
     and gets a chunk of min(tokens left, budget left, its side's share).  A scanner stops at its
     first refusal or when its share is spent.
  4. Second pass: what is left of the budget is offered to the waiting requests of step 2, then to
     both scanners again without the per-side limits (memory: used[0] + used[1] + need <= M).
  5. Steps of more than `row_multiple` rows are cut to a multiple of it, the surplus taken off the
     prefill chunks at the end of the list (Appendix A.2: batch sizes in multiples of 128).
  6. The descriptor: prefill segments in the order of the list, decode sequences in leaf order;
     prefix nodes = segments with at least two decode members in this step and at least one page,
     in DFS order; page tables carry the physical pages (shared pages first, root to leaf).
  7. Commit: prefill chunks advance `cached` and mark the segments they cover as computed; a
     request whose prompt is complete has produced its first token; decode rows add one token; a
     request past its estimate is charged one more token per step and, if it was admitted from
     the left and generated * 100 >= relocate_pct * d_est, moves with its own reservation to the
     right partition; a request that has produced d_true tokens leaves and frees its pages.
"""
from __future__ import annotations

import heapq
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

PS = 16


class _Live:
    __slots__ = ("req", "side", "cached", "generated", "reserved", "pages")

    def __init__(self, req, side, cached):
        self.req, self.side, self.cached = req, side, cached
        self.generated, self.reserved, self.pages = 0, 0, []


class SchedulerOracle:
    def __init__(self, tree, d_true: Sequence[int], mem_tokens: int, token_budget: int, n_pages: int,
                 order: Optional[Sequence[int]] = None, relocate_pct: int = 200, row_multiple: int = 1):
        """tree: a finalized oracle.builder.BuilderOracle (requests with n_cached = 0)."""
        self.t = tree
        self.reqs = tree.reqs
        self.d_true = [int(d) for d in d_true]
        self.mem_tokens, self.token_budget, self.n_pages = int(mem_tokens), int(token_budget), int(n_pages)
        self.relocate_pct, self.row_multiple = int(relocate_pct), max(1, int(row_multiple))
        nodes = tree.nodes
        self.leaf = {nd.req: i for i, nd in enumerate(nodes) if nd.req >= 0}
        self.pos_in_leaf_order = {r: k for k, r in enumerate(tree.leaf_order)}
        self.two_sided = order is None
        if order is None:
            self.order = list(tree.leaf_order)
            b = tree.budgets()
            m = b["m_l"] + b["m_r"]
            frac_l = b["m_l"] / m if m > 0 else 0.5
            cap_l = int(np.floor(float(self.mem_tokens) * frac_l))
            self.cap = [cap_l, self.mem_tokens - cap_l]
            c_l, c_r = b["c_l"], b["c_r"]
            self.pre_num, self.pre_den = (1, 2) if (c_l < 0 or c_r < 0 or c_l + c_r == 0) else (c_l, c_l + c_r)
            _, L, R = tree.scan_sides()
            self.p_side = [-(-tree.nodes[x].sum_p // tree.nodes[x].n_req) for x in (L, R)]
        else:
            self.order = [int(r) for r in order]
            self.cap = [self.mem_tokens, 0]
            self.pre_num, self.pre_den = 1, 1
            self.p_side = [0, 0]
        self.lo, self.hi = 0, len(self.order) - 1
        # shareable pages of every internal node
        n = len(nodes)
        self.page_lo, self.page_hi = [0] * n, [0] * n
        for i in tree.dfs:                                 # parents before children
            nd = nodes[i]
            if nd.req >= 0:
                continue
            above = self.page_hi[nd.parent] if nd.parent >= 0 else 0
            ends_here = any(nodes[c].req >= 0 and nodes[c].end == nd.end for c in nd.children)
            hi = (nd.end - 1) // PS if (ends_here and nd.end > 0) else nd.end // PS
            self.page_lo[i], self.page_hi[i] = above, max(above, hi)
        self.ref, self.done, self.owner, self.nside = [0] * n, [0] * n, [-1] * n, [0] * n
        self.node_pages: Dict[int, List[int]] = {}
        self.live: Dict[int, _Live] = {}
        self.admitted: List[int] = []
        self.used = [0, 0]
        self.free = list(range(self.n_pages))
        heapq.heapify(self.free)
        self.stats = dict(steps=0, rows=0, prefill_rows=0, decode_rows=0, prompt_tokens_skipped=0, tokens_out=0,
                          finished=0, peak_tokens=0, peak_pages=0, relocated=0)

    # -- tree helpers ---------------------------------------------------------------------
    def path(self, r: int) -> List[int]:
        """Internal ancestors of request r with a non-empty segment, top down."""
        out = []
        n = self.t.nodes[self.leaf[r]].parent
        while n >= 0:
            if self.t.nodes[n].end > self.t.nodes[n].start:
                out.append(n)
            n = self.t.nodes[n].parent
        out.reverse()
        return out

    def shared_hi(self, r: int) -> int:
        p = self.path(r)
        return self.page_hi[p[-1]] if p else 0

    def _take_page(self) -> int:
        if not self.free:
            raise MemoryError("the page pool is exhausted")
        return heapq.heappop(self.free)

    # -- admission ------------------------------------------------------------------------
    def _try_admit(self, r: int, side: int, borrow: bool) -> Optional[_Live]:
        nodes = self.t.nodes
        p = len(self.reqs[r].tokens)
        path = self.path(r)
        cached_pages, chain, mine = 0, True, []
        for n in path:
            seg = nodes[n].end - nodes[n].start
            if self.ref[n] > 0 and self.done[n] == seg:
                if chain:
                    cached_pages = self.page_hi[n]
            elif self.ref[n] > 0 and self.owner[n] >= 0:
                return None                              # somebody is still computing this segment
            else:
                mine.append(n)
                chain = False
        own = (p - nodes[self.leaf[r]].start) + int(self.reqs[r].d_est)
        need = own + sum(nodes[n].end - nodes[n].start for n in path if self.ref[n] == 0)
        over = (self.used[0] + self.used[1] + need > self.mem_tokens) if borrow else (self.used[side] + need > self.cap[side])
        if over and self.live:
            return None
        lv = _Live(r, side, min(PS * cached_pages, p - 1))
        lv.reserved = own
        self.used[side] += own
        for n in path:
            if self.ref[n] == 0:
                self.used[side] += nodes[n].end - nodes[n].start
                self.nside[n], self.done[n], self.owner[n] = side, 0, -1
                self.node_pages[n] = []
            self.ref[n] += 1
        for n in mine:
            self.owner[n] = r
        self.stats["prompt_tokens_skipped"] += lv.cached
        self.live[r] = lv
        self.admitted.append(r)
        return lv

    def _release(self, lv: _Live):
        nodes = self.t.nodes
        self.used[lv.side] -= lv.reserved
        for pg in lv.pages:
            heapq.heappush(self.free, pg)
        for n in self.path(lv.req):
            self.ref[n] -= 1
            if self.ref[n] == 0:
                self.used[self.nside[n]] -= nodes[n].end - nodes[n].start
                self.done[n], self.owner[n] = 0, -1
                for pg in self.node_pages.pop(n, []):
                    heapq.heappush(self.free, pg)
        del self.live[lv.req]

    @property
    def finished(self) -> bool:
        return not self.live and self.lo > self.hi

    # -- one step ---------------------------------------------------------------------------
    def plan(self):
        budget = self.token_budget
        dec = [(lv.req, len(self.reqs[lv.req].tokens) + lv.generated - 1)
               for lv in self.live.values() if lv.cached >= len(self.reqs[lv.req].tokens)]
        dec.sort(key=lambda x: self.pos_in_leaf_order[x[0]])
        budget -= len(dec)
        pre: List[Tuple[int, int, int]] = []
        self.admitted = [r for r in self.admitted if r in self.live and self.live[r].cached < len(self.reqs[r].tokens)]
        b0 = max(0, budget)
        left = b0 * self.pre_num // self.pre_den
        if self.two_sided:
            left = max(left, min(self.p_side[0], b0 // 2))
            left = min(left, b0 - min(self.p_side[1], b0 // 2))
        share = [left, b0 - left]
        waiting = []
        for r in self.admitted:
            lv = self.live[r]
            chunk = min(len(self.reqs[r].tokens) - lv.cached, share[lv.side])
            if chunk <= 0:
                waiting.append(r)
                continue
            pre.append((r, lv.cached, chunk))
            budget -= chunk
            share[lv.side] -= chunk
        for borrow in (False, True):
            is_open = [True, self.two_sided]
            if borrow:
                for r in waiting:
                    if budget <= 0:
                        break
                    lv = self.live[r]
                    chunk = min(len(self.reqs[r].tokens) - lv.cached, budget)
                    pre.append((r, lv.cached, chunk))
                    budget -= chunk
                share = [budget, budget]
            while budget > 0 and self.lo <= self.hi and (is_open[0] or is_open[1]):
                progressed = False
                for side in (0, 1):
                    if not is_open[side] or self.lo > self.hi or budget <= 0:
                        continue
                    if share[side] <= 0:
                        is_open[side] = False
                        continue
                    r = self.order[self.lo] if side == 0 else self.order[self.hi]
                    lv = self._try_admit(r, side, borrow)
                    if lv is None:
                        is_open[side] = False
                        continue
                    if side == 0:
                        self.lo += 1
                    else:
                        self.hi -= 1
                    chunk = min(len(self.reqs[r].tokens) - lv.cached, budget, share[side])
                    pre.append((r, lv.cached, chunk))
                    budget -= chunk
                    share[side] -= chunk
                    progressed = True
                if not progressed:
                    break
        total = len(dec) + sum(c for _, _, c in pre)
        extra = total % self.row_multiple if total > self.row_multiple else 0
        while extra > 0 and pre:
            r, cached, chunk = pre[-1]
            cut = min(extra, chunk)
            if cut == chunk:
                pre.pop()
            else:
                pre[-1] = (r, cached, chunk - cut)
            extra -= cut
        return pre, dec

    def _page_of(self, lv: _Live, j: int, may_allocate: bool) -> int:
        """Physical page of logical page j of a live request."""
        sh = self.shared_hi(lv.req)
        if j < sh:
            for n in self.path(lv.req):
                if self.page_lo[n] <= j < self.page_hi[n]:
                    pages = self.node_pages[n]
                    k = j - self.page_lo[n]
                    while may_allocate and len(pages) <= k:
                        pages.append(self._take_page())
                    return pages[k]
            raise AssertionError("no node owns a shared page")
        k = j - sh
        while may_allocate and len(lv.pages) <= k:
            lv.pages.append(self._take_page())
        return lv.pages[k]

    def emit(self, pre, dec):
        nodes = self.t.nodes
        # pages that this step writes into come into being, in the order of the descriptor
        for r, cached, chunk in pre:
            for j in range(cached // PS, (cached + chunk - 1) // PS + 1):
                self._page_of(self.live[r], j, True)
        for r, ctx in dec:
            self._page_of(self.live[r], ctx // PS, True)
        row_start, kv_len, page_start, page_ids, seq_leaf, seq_req = [0], [], [0], [], [], []
        for r, cached, chunk in pre:
            kv = cached + chunk
            page_ids.extend(self._page_of(self.live[r], j, False) for j in range(-(-kv // PS)))
            row_start.append(row_start[-1] + chunk)
            kv_len.append(kv); page_start.append(len(page_ids)); seq_leaf.append(-1); seq_req.append(r)
        members: Dict[int, List[int]] = {}
        for k, (r, ctx) in enumerate(dec):
            for n in self.path(r):
                members.setdefault(n, []).append(k)
        node_id: Dict[int, int] = {}
        node_parent, node_first, node_count, node_page_start, node_page_ids = [], [], [], [0], []
        for n in self.t.dfs:
            m = members.get(n, [])
            if nodes[n].req >= 0 or len(m) < 2 or self.page_hi[n] <= self.page_lo[n]:
                continue
            anc = nodes[n].parent
            while anc >= 0 and anc not in node_id:
                anc = nodes[anc].parent
            node_id[n] = len(node_parent)
            node_parent.append(node_id[anc] if anc >= 0 else -1)
            node_first.append(len(pre) + min(m))
            node_count.append(len(m))
            node_page_ids.extend(self.node_pages[n])
            node_page_start.append(len(node_page_ids))
        for r, ctx in dec:
            kv = ctx + 1
            page_ids.extend(self._page_of(self.live[r], j, False) for j in range(-(-kv // PS)))
            row_start.append(row_start[-1] + 1)
            deepest = -1
            for n in self.path(r):
                if n in node_id:
                    deepest = node_id[n]
            kv_len.append(kv); page_start.append(len(page_ids)); seq_leaf.append(deepest); seq_req.append(r)
        i32 = lambda a: np.asarray(a, dtype=np.int32)
        return dict(n_seq=len(pre) + len(dec), n_prefill=len(pre), n_rows=row_start[-1], row_start=i32(row_start),
                    kv_len=i32(kv_len), page_start=i32(page_start), page_ids=i32(page_ids), n_nodes=len(node_parent),
                    node_parent=i32(node_parent), node_page_start=i32(node_page_start), node_page_ids=i32(node_page_ids),
                    node_seq_first=i32(node_first), node_seq_count=i32(node_count), seq_leaf_node=i32(seq_leaf),
                    seq_request=i32(seq_req), n_pages=self.n_pages)

    def commit(self, pre, dec):
        nodes, st = self.t.nodes, self.stats
        st["steps"] += 1
        st["prefill_rows"] += sum(c for _, _, c in pre)
        st["decode_rows"] += len(dec)
        st["rows"] += sum(c for _, _, c in pre) + len(dec)
        st["peak_tokens"] = max(st["peak_tokens"], self.used[0] + self.used[1])
        st["peak_pages"] = max(st["peak_pages"], self.n_pages - len(self.free))
        for r, cached, chunk in pre:
            lv = self.live[r]
            lo, hi = cached, cached + chunk
            for n in self.path(r):
                s, e = nodes[n].start, nodes[n].end
                if hi <= s or lo >= e or self.owner[n] != r:
                    continue
                self.done[n] = max(self.done[n], min(hi, e) - s)
                if self.done[n] == e - s:
                    self.owner[n] = -1
            lv.cached = hi
            if lv.cached == len(self.reqs[r].tokens):
                lv.generated = 1
                st["tokens_out"] += 1
                if lv.generated >= self.d_true[r]:
                    st["finished"] += 1
                    self._release(lv)
        for r, ctx in dec:
            lv = self.live[r]
            lv.generated += 1
            st["tokens_out"] += 1
            d_est = int(self.reqs[r].d_est)
            if lv.generated > d_est:
                lv.reserved += 1
                self.used[lv.side] += 1
                if self.two_sided and lv.side == 0 and self.relocate_pct > 0 and lv.generated * 100 >= self.relocate_pct * d_est:
                    self.used[0] -= lv.reserved
                    self.used[1] += lv.reserved
                    lv.side = 1
                    st["relocated"] += 1
            if lv.generated >= self.d_true[r]:
                st["finished"] += 1
                self._release(lv)

    def next_step(self):
        """The descriptor of the next step (state already advanced past it), or None when the pool is served."""
        if self.finished:
            return None
        pre, dec = self.plan()
        if not pre and not dec:
            raise RuntimeError("the driver is stuck: nothing fits the memory of either side")
        d = self.emit(pre, dec)
        self.commit(pre, dec)
        return d
