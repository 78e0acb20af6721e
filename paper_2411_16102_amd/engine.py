"""A pool of requests served to completion through the blended step: glue only.

The method's runtime scheduling - request state, the two scanners, the memory partition, chunked
prefill budgets, the adaptation to misjudged output lengths, the runtime prefix tree and the page
allocator (BlendServe Sections 3.2, 5.3, 5.4, Appendix A.2) - lives in the library behind
`bs_sched_*` (csrc/builder.cpp).  This module builds the library objects for a pool, loops
`Scheduler.next_step` -> `bs_blend_step`, and adds up device time.  The KV pool is one tensor that
persists over the steps: the scheduler's pages are physical, so what a prefill chunk appends in
one step is what the decode rows of later steps attend to.
"""
from __future__ import annotations

from typing import Callable, Optional, Sequence

import numpy as np

from . import workloads as W


def make_scheduler(api, reqs: Sequence[W.PoolRequest], hw: dict, mem_tokens: int, token_budget: int, n_pages: int,
                   policy: str = "blend", seed: int = 0, split_t: int = 0, split_budget: int = -1,
                   mem_model: str = "expanded", relocate_pct: int = 200, row_multiple: int = 1):
    """(builder, scheduler, split info) for a pool.  policy: "blend" = the sorted (and optionally split)
    resource-aware tree scanned from both ends; "dfs" / "random" = that order walked from the left."""
    b = api.Builder(hw["p_model"], hw["kv_bytes"], hw["compute"], hw["bandwidth"], mem_tokens * hw["kv_bytes"], 16)
    if mem_model != "expanded":
        b.set_mem_model(mem_model)
        split_t = 0                       # node splitting is defined for the additive model
    for r in reqs:
        b.add(r.tokens, r.d_est, 0)
    b.finalize()
    split_info = b.split(split_t, split_budget) if (policy == "blend" and split_t > 0) else None
    order = None if policy == "blend" else W.baseline_order(reqs, policy, seed)
    s = api.Scheduler(b, [r.d_true for r in reqs], mem_tokens, token_budget, n_pages, order=order,
                      relocate_pct=relocate_pct if policy == "blend" else 0, row_multiple=row_multiple)
    return b, s, split_info


def serve(sched, step_fn: Callable[[dict], None], progress: Optional[Callable[[dict], None]] = None, max_steps: int = 10 ** 7):
    """Runs every step of the pool through step_fn(descriptor); returns the scheduler's statistics."""
    n = 0
    while n < max_steps:
        d = sched.next_step()
        if d is None:
            break
        step_fn(d)
        n += 1
        if progress and n % 200 == 0:
            progress(sched.stats())
    return sched.stats()


class GpuStepper:
    """Runs descriptors through bs_blend_step on one layer of the given shape, over ONE persistent KV
    pool, and adds up the device time of the steps (HIP events on the stream, read back at the end).
    x of a step: rows of a fixed seeded tensor (row i of the step takes row i): the driver is timed
    and its numerics are checked elsewhere against the oracle chain with the same inputs."""

    def __init__(self, api, shape, max_rows: int, pool_pages: int, seed: int = 0, flags: int = 0):
        import torch
        self.torch = torch
        self.layer = api.Layer(shape, device=0)
        probe = W.assemble_batch(16, [(1, 1, -1)], 0, [], None)
        tens = W.make_tensors(shape, probe, seed)
        self.weights, self.keep = self.layer.upload_weights(tens)
        g = torch.Generator(device="cuda").manual_seed(seed)
        self.x = torch.randn((max_rows, shape.d_model), device="cuda", generator=g).to(torch.bfloat16)
        self.y = torch.empty_like(self.x)
        self.pool_pages = int(pool_pages)
        self.pool = torch.zeros((self.pool_pages * self.layer.page_bytes() // 2,), device="cuda", dtype=torch.bfloat16)
        self.events = []
        self.api = api
        self.flags = flags

    def __call__(self, d: dict):
        import ctypes as C
        torch = self.torch
        if d["n_pages"] > self.pool_pages or d["n_rows"] > self.x.shape[0]:
            raise RuntimeError("step of %d rows / %d pages exceeds the stepper's buffers" % (d["n_rows"], d["n_pages"]))
        batch = W.Batch(page_size=16, **{k: v for k, v in d.items() if k != "seq_request"})
        desc, keep = self.api.marshal_batch(batch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        lay = self.layer
        lay._check(lay.lib.bs_blend_step(lay.h, C.byref(self.weights), C.byref(desc), C.c_void_p(self.x.data_ptr()),
                                         C.c_void_p(self.y.data_ptr()), C.c_void_p(self.pool.data_ptr()), self.pool_pages,
                                         lay._stream(None), self.flags))
        e1.record()
        self.events.append((e0, e1))

    def total_ms(self) -> float:
        self.torch.cuda.synchronize()
        return float(sum(a.elapsed_time(b) for a, b in self.events))
