"""Multi-step driver: a pool of requests served to completion through the blended step.

BlendServe (Sections 3.2, 5.3, Appendix A.2) re-forms the runtime batch every iteration
from the requests in flight: decoding requests contribute one row each, the rest of the
token budget goes to prefill chunks, and new requests are admitted from the two ends of the
density-sorted leaf order (one scanner per end, the KV memory split between them by
Algorithm 3) as memory allows.  This module is that loop, with three admission orders so
that the effect of the order can be measured on one GPU (the ablation of Section 6.3:
resource-aware order against prefix-DFS order and against a random order):

  blend   leaf order of the sorted (and optionally split) resource-aware prefix tree,
          scanned from both ends;
  dfs     prompts in lexicographic order, i.e. DFS order of the plain prefix tree (best
          prefix sharing), scanned from the left;
  random  a seeded permutation, scanned from the left.

The driver keeps request state (tokens cached, tokens generated) and the memory account
itself and asks the library's builder for the descriptor of each step (`Builder.emit`).
Pages are numbered afresh every step, so the KV contents carry no meaning from step to
step: the driver measures time and token counts, not outputs (the step's numerics are
tested against the oracle elsewhere).  Prefix sharing is honoured in three places: a shared
prompt segment is computed by the first resident request that needs it and skipped by the
others (a request whose prefix is still being computed by another waits), its KV is
counted once in the memory account while any sharer is resident, and the descriptor's
prefix nodes let decode attention read it once per group.

Output lengths: the order and the memory reservation use the estimate `d_est`; a request
finishes after `d_true` tokens.  The batch adapts to misjudged lengths as Section 5.4 describes:
a request that ends early frees its reservation at once and the scanners admit others in its
place; one that runs past its estimate has its account grow token by token; and one admitted
from the compute-intensive end whose output has grown to `relocate_factor` times its estimate
(a severe underestimate: it is a memory-intensive request after all) is moved, with its own
reservation, from the left memory partition to the right one, so that the left scanner gets its
share back for the requests it is meant to admit.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class PoolRequest:
    tokens: Sequence[int]
    d_est: int
    d_true: int


@dataclass
class _Live:
    req: int
    side: int              # 0 = left scanner, 1 = right scanner
    cached: int            # prompt tokens whose KV exists (own or shared)
    generated: int = 0
    reserved: int = 0      # tokens charged to the memory account for this request alone


class Engine:
    def __init__(self, builder, requests: Sequence[PoolRequest], mem_tokens: int, policy: str = "blend",
                 token_budget: int = 2560, split_t: int = 0, split_budget: int = -1, seed: int = 0,
                 mem_model: str = "expanded", relocate_factor: float = 2.0, row_multiple: int = 1):
        assert policy in ("blend", "dfs", "random")
        self.relocate_factor = float(relocate_factor)   # 0: requests stay on the side that admitted them
        self.row_multiple = max(1, int(row_multiple))   # steps of more rows than this are cut to a multiple of it
        if mem_model != "expanded":
            builder.set_mem_model(mem_model)   # densities with shared prefix pages read once per step
            split_t = 0                        # node splitting is defined for the additive model
        self.b = builder
        self.reqs = list(requests)
        self.policy = policy
        self.mem_tokens = int(mem_tokens)
        self.token_budget = int(token_budget)
        for r in self.reqs:
            builder.add(r.tokens, r.d_est, 0)
        builder.finalize()
        self.split_info = builder.split(split_t, split_budget) if (policy == "blend" and split_t > 0) else None
        t = builder.tree()
        self.parent, self.start, self.end, self.node_req = t["parent"], t["start"], t["end"], t["req"]
        n_nodes = len(self.parent)
        self.leaf_node = np.full(len(self.reqs), -1, dtype=np.int64)
        for n in range(n_nodes):
            if self.node_req[n] >= 0:
                self.leaf_node[self.node_req[n]] = n
        if policy == "blend":
            self.order = [int(r) for r in t["leaf_order"]]
            info, _ = builder.next_batch()
            m = float(info["m_l"]) + float(info["m_r"])
            frac_l = float(info["m_l"]) / m if m > 0 else 0.5
            # a side never gets less than a twentieth of the memory: its scanner must be able to move
            frac_l = min(max(frac_l, 0.05), 0.95)
            self.cap = [int(self.mem_tokens * frac_l), self.mem_tokens - int(self.mem_tokens * frac_l)]
            c_l, c_r = info["c_l"], info["c_r"]
            if c_l < 0 or c_r < 0 or c_l + c_r == 0:
                self.pre_frac_l = 0.5
            else:
                self.pre_frac_l = min(max(c_l / float(c_l + c_r), 0.1), 0.9)
        else:
            if policy == "dfs":
                self.order = sorted(range(len(self.reqs)), key=lambda i: (list(self.reqs[i].tokens), i))
            else:
                self.order = [int(i) for i in np.random.default_rng(seed).permutation(len(self.reqs))]
            self.cap = [self.mem_tokens, 0]
            self.pre_frac_l = 1.0
        self.lo, self.hi = 0, len(self.order) - 1     # next candidates of the two scanners
        self.live: Dict[int, _Live] = {}
        self.admitted: List[int] = []                 # admission order of live prefilling requests
        self.used = [0, 0]                            # tokens charged per side
        # shared prompt segments: residents below, tokens computed, who computes them
        self.node_ref = np.zeros(n_nodes, dtype=np.int64)
        self.node_done = np.zeros(n_nodes, dtype=np.int64)
        self.node_owner = np.full(n_nodes, -1, dtype=np.int64)
        self.node_side = np.zeros(n_nodes, dtype=np.int64)
        self.stats = dict(steps=0, rows=0, prefill_rows=0, decode_rows=0, prompt_tokens_skipped=0, tokens_out=0,
                          finished=0, peak_tokens=0, kv_tokens_read=0, relocated=0)

    # -- helpers ---------------------------------------------------------------------------
    def _path(self, r: int) -> List[int]:
        """Internal nodes from the root's child down to the leaf's parent (shared segments)."""
        out = []
        n = int(self.parent[self.leaf_node[r]])
        while n > 0:
            out.append(n)
            n = int(self.parent[n])
        out.reverse()
        return out

    def _try_admit(self, r: int, side: int, borrow: bool = False) -> Optional[_Live]:
        req = self.reqs[r]
        p = len(req.tokens)
        path = self._path(r)
        cached = 0
        mine = []                                # segments this request would have to compute itself
        for n in path:
            seg = int(self.end[n] - self.start[n])
            if self.node_ref[n] > 0 and self.node_done[n] == seg:
                if cached == int(self.start[n]):
                    cached = int(self.end[n])    # resident and complete: nothing to compute
            elif self.node_ref[n] > 0 and self.node_owner[n] >= 0:
                return None                      # another request is still computing this segment
            else:
                mine.append(n)
        need = (p - int(self.start[self.leaf_node[r]])) + int(req.d_est)     # own segment + output
        for n in path:
            if self.node_ref[n] == 0:
                need += int(self.end[n] - self.start[n])
        # a side keeps to its share of the memory (Algorithm 3) unless the other side has left some unused
        over = (self.used[0] + self.used[1] + need > self.mem_tokens) if borrow else (self.used[side] + need > self.cap[side])
        if over and self.live:
            return None
        lv = _Live(r, side, cached)
        own = (p - int(self.start[self.leaf_node[r]])) + int(req.d_est)
        lv.reserved = own
        self.used[side] += own
        for n in path:
            if self.node_ref[n] == 0:
                self.used[side] += int(self.end[n] - self.start[n])
                self.node_side[n] = side
                self.node_done[n] = 0
                self.node_owner[n] = -1
            self.node_ref[n] += 1
        for n in mine:
            self.node_owner[n] = r
        self.stats["prompt_tokens_skipped"] += cached
        self.live[r] = lv
        self.admitted.append(r)
        return lv

    def _release(self, lv: _Live):
        self.used[lv.side] -= lv.reserved
        for n in self._path(lv.req):
            self.node_ref[n] -= 1
            if self.node_ref[n] == 0:
                self.used[int(self.node_side[n])] -= int(self.end[n] - self.start[n])
                self.node_done[n] = 0
                self.node_owner[n] = -1
        del self.live[lv.req]

    def _advance_prefill(self, lv: _Live, chunk: int):
        """Mark the shared segments covered by [cached, cached + chunk) as computed."""
        lo, hi = lv.cached, lv.cached + chunk
        for n in self._path(lv.req):
            s, e = int(self.start[n]), int(self.end[n])
            if hi <= s or lo >= e:
                continue
            if self.node_owner[n] == lv.req:
                self.node_done[n] = max(int(self.node_done[n]), min(hi, e) - s)
                if self.node_done[n] == e - s:
                    self.node_owner[n] = -1
        lv.cached = hi

    @property
    def done(self) -> bool:
        return not self.live and self.lo > self.hi

    # -- one iteration ----------------------------------------------------------------------
    def plan_step(self):
        """Returns (pre, dec): the explicit step for Builder.emit, or None when the pool is done."""
        if self.done:
            return None
        budget = self.token_budget
        dec = [(lv.req, len(self.reqs[lv.req].tokens) + lv.generated - 1)
               for lv in self.live.values() if lv.cached >= len(self.reqs[lv.req].tokens)]
        budget -= len(dec)
        pre: List[Tuple[int, int, int]] = []
        self.admitted = [r for r in self.admitted if r in self.live and self.live[r].cached < len(self.reqs[r].tokens)]
        # the prefill budget of the step is shared between the sides as Algorithm 3 says (C_L : C_R);
        # chunks of requests already being prefilled draw on their side's share first
        side_budget = [int(budget * self.pre_frac_l), budget - int(budget * self.pre_frac_l)]
        waiting = []
        for r in self.admitted:
            lv = self.live[r]
            chunk = min(len(self.reqs[r].tokens) - lv.cached, side_budget[lv.side])
            if chunk <= 0:
                waiting.append(r)
                continue
            pre.append((r, lv.cached, chunk))
            budget -= chunk
            side_budget[lv.side] -= chunk
        for borrow in (False, True):
            # second pass: what one side could not use (memory, prefill budget) is offered to the other
            open_side = [True, self.policy == "blend"]
            if borrow:
                side_budget = [budget, budget]
                for r in waiting:                     # started requests come before new ones
                    if budget <= 0:
                        break
                    lv = self.live[r]
                    chunk = min(len(self.reqs[r].tokens) - lv.cached, budget)
                    pre.append((r, lv.cached, chunk))
                    budget -= chunk
                side_budget = [budget, budget]
            while budget > 0 and self.lo <= self.hi and (open_side[0] or open_side[1]):
                progressed = False
                for side in (0, 1):
                    if not open_side[side] or self.lo > self.hi or budget <= 0:
                        continue
                    if side_budget[side] <= 0:
                        open_side[side] = False
                        continue
                    r = self.order[self.lo] if side == 0 else self.order[self.hi]
                    lv = self._try_admit(r, side, borrow)
                    if lv is None:
                        open_side[side] = False
                        continue
                    if side == 0:
                        self.lo += 1
                    else:
                        self.hi -= 1
                    p = len(self.reqs[r].tokens)
                    if lv.cached >= p:                # whole prompt shared and computed: one row recomputes the last token
                        lv.cached = p - 1
                        self.stats["prompt_tokens_skipped"] -= 1
                    chunk = min(p - lv.cached, budget, side_budget[side])
                    pre.append((r, lv.cached, chunk))
                    budget -= chunk
                    side_budget[side] -= chunk
                    progressed = True
                if not progressed:
                    break
        # Batch sizes in multiples of `row_multiple` (128 in Appendix A.2; off by default here: on
        # this library's GEMMs, which pick their tile shape per row count, it changed nothing for the
        # resource-aware order and cost the DFS order 1.5 % through the extra steps).  The surplus
        # rows come off the prefill chunks at the end of the list (newest first) and are computed
        # in the next step.
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

    def commit_step(self, pre, dec):
        st = self.stats
        st["steps"] += 1
        st["prefill_rows"] += sum(c for _, _, c in pre)
        st["decode_rows"] += len(dec)
        st["rows"] += sum(c for _, _, c in pre) + len(dec)
        st["peak_tokens"] = max(st["peak_tokens"], self.used[0] + self.used[1])
        st["kv_tokens_read"] += sum(ctx + 1 for _, ctx in dec)
        for r, _, chunk in pre:
            lv = self.live[r]
            self._advance_prefill(lv, chunk)
            if lv.cached == len(self.reqs[r].tokens):
                lv.generated = 1                      # the last prompt row yields the first output token
                st["tokens_out"] += 1
                if lv.generated >= self.reqs[r].d_true:
                    st["finished"] += 1
                    self._release(lv)
        for r, _ in dec:
            lv = self.live[r]
            lv.generated += 1
            st["tokens_out"] += 1
            if lv.generated > self.reqs[r].d_est:     # ran past its estimate: the account follows
                lv.reserved += 1
                self.used[lv.side] += 1
                if (self.policy == "blend" and lv.side == 0 and self.relocate_factor > 0
                        and lv.generated >= self.relocate_factor * self.reqs[r].d_est):
                    # severely underestimated (Section 5.4): from the left partition to the right one
                    self.used[0] -= lv.reserved
                    self.used[1] += lv.reserved
                    lv.side = 1
                    st["relocated"] += 1
            if lv.generated >= self.reqs[r].d_true:
                st["finished"] += 1
                self._release(lv)

    # -- the whole pool ---------------------------------------------------------------------
    def run(self, step_fn: Callable[[dict], None], progress: Optional[Callable[[dict], None]] = None, max_steps: int = 10 ** 7):
        """step_fn(descriptor) executes (or prices) one step."""
        while not self.done and self.stats["steps"] < max_steps:
            plan = self.plan_step()
            if plan is None:
                break
            pre, dec = plan
            if not pre and not dec:
                raise RuntimeError("the driver is stuck: nothing fits the memory of either side")
            step_fn(self.b.emit(pre, dec))
            self.commit_step(pre, dec)
            if progress and self.stats["steps"] % 200 == 0:
                progress(self.stats)
        return self.stats


class GpuStepper:
    """Runs descriptors through bs_blend_step on one layer of the given shape and adds up the
    device time of the steps (HIP events on the stream, read back once at the end)."""

    def __init__(self, api, shape, max_rows: int, pool_pages: int, seed: int = 0):
        import torch
        from . import workloads as W
        self.torch, self.W = torch, W
        self.layer = api.Layer(shape, device=0)
        probe = W.assemble_batch(16, [(1, 1, -1)], 0, [], None)
        tens = W.make_tensors(shape, probe, seed)
        self.weights, self.keep = self.layer.upload_weights(tens)
        g = torch.Generator(device="cuda").manual_seed(seed)
        self.x = torch.randn((max_rows, shape.d_model), device="cuda", generator=g).to(torch.bfloat16)
        self.y = torch.empty_like(self.x)
        self.pool_pages = int(pool_pages)
        self.pool = (torch.randn((self.pool_pages * self.layer.page_bytes() // 2,), device="cuda", generator=g) * 0.5).to(torch.bfloat16)
        self.events = []
        self.api = api

    def __call__(self, d: dict):
        import ctypes as C
        torch = self.torch
        if d["n_pages"] > self.pool_pages or d["n_rows"] > self.x.shape[0]:
            raise RuntimeError("step of %d rows / %d pages exceeds the stepper's buffers" % (d["n_rows"], d["n_pages"]))
        batch = self.W.Batch(page_size=16, **{k: v for k, v in d.items() if k != "seq_request"})
        desc, keep = self.api.marshal_batch(batch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        lay = self.layer
        lay._check(lay.lib.bs_blend_step(lay.h, C.byref(self.weights), C.byref(desc), C.c_void_p(self.x.data_ptr()),
                                         C.c_void_p(self.y.data_ptr()), C.c_void_p(self.pool.data_ptr()), self.pool_pages,
                                         lay._stream(None), 0))
        e1.record()
        self.events.append((e0, e1))

    def total_ms(self) -> float:
        self.torch.cuda.synchronize()
        return float(sum(a.elapsed_time(b) for a, b in self.events))


def synthetic_pool(seed: int, n_groups: int = 24, per_group: int = 12, n_fresh: int = 96, est_noise: float = 0.25) -> List[PoolRequest]:
    """A pool with the structure of the paper's mixed workloads (Section 6.1): groups sharing a
    long system prompt whose members generate short outputs (compute-intensive, benchmark-like),
    groups with medium and with long outputs (memory-intensive), and unrelated prompt-heavy
    requests.  Each kind comes from its own dataset, whose prompts start with the same template
    token, so the prefix-DFS order serves one dataset after the other, as it would a concatenation
    of traces; the template tokens are numbered so that it meets the compute-intensive datasets
    first and the long-output one last (the order that hurts it: Section 3.1).  Output-length
    estimates are the true lengths with multiplicative noise."""
    rng = np.random.default_rng(seed)
    out: List[PoolRequest] = []
    for g in range(n_groups):
        kind = g % 3
        prefix = [kind + 1] + [int(t) for t in rng.integers(4, 128000, int(rng.integers(256, 1536)))]
        for _ in range(per_group):
            own = [int(t) for t in rng.integers(4, 128000, int(rng.integers(16, 256)))]
            d = int(rng.integers(8, 48)) if kind == 0 else int(rng.integers(128, 512)) if kind == 1 else int(rng.integers(768, 2048))
            out.append(PoolRequest(prefix + own, 0, d))
    for _ in range(n_fresh):
        toks = [0] + [int(t) for t in rng.integers(4, 128000, int(rng.integers(512, 3072)))]
        out.append(PoolRequest(toks, 0, int(rng.integers(4, 64))))
    for r in out:
        r.d_est = max(1, int(round(r.d_true * float(np.exp(est_noise * rng.standard_normal())))))
    perm = rng.permutation(len(out))
    return [out[i] for i in perm]
