"""The multi-step driver on the GPU.  A small pool is served to completion through bs_blend_step over
ONE KV pool that persists from step to step (the scheduler's pages are physical): every step's
descriptor must equal the oracle scheduler's bit for bit, and every step's output must match the
oracle chain - the layer oracle applied step after step to its own copy of the pool, into which it
appends its own keys and values - within the tolerance rule.  What a prefill chunk appends in one step
is what later steps attend to, so a page that moved, was freed too early or was shared wrongly shows up
as a wrong output."""
import dataclasses

import numpy as np
import pytest

from oracle import builder as OB
from oracle import layer as O
from oracle import scheduler as OS
from paper_2411_16102_amd import engine as E, workloads as W
from parity_rule import check

pytestmark = pytest.mark.gpu

HW = dict(p_model=8_030_000_000, kv_bytes=512, compute=2.5e15, bandwidth=8.0e12)


def small_pool(seed):
    rng = np.random.default_rng(seed)
    reqs = []
    for g in range(3):
        prefix = [int(t) for t in rng.integers(10, 5000, int(rng.choice([32, 40, 64])))]
        for k in range(4):
            own = [int(t) for t in rng.integers(10, 5000, int(rng.integers(1, 30)))]
            d = int(rng.choice([1, 2, 4, 7]))
            reqs.append(W.PoolRequest(prefix + own, max(1, d + int(rng.integers(-1, 3))), d))
    for _ in range(5):
        reqs.append(W.PoolRequest([int(t) for t in rng.integers(10, 5000, int(rng.integers(8, 90)))], 2, int(rng.choice([1, 3]))))
    reqs.append(W.PoolRequest(list(reqs[0].tokens), 3, 3))        # an exact duplicate
    return reqs


@pytest.mark.parametrize("seed,flags", [(0, 0), (1, 0), (2, 1)])
def test_pool_outputs_match_the_oracle_chain_step_by_step(lib, seed, flags):
    import torch
    shape = W.TINY
    reqs = small_pool(seed)
    mem, budget, pages = 420, 80, 72
    b, sched, _ = E.make_scheduler(lib, reqs, HW, mem, budget, pages, policy="blend")
    cm = OB.CostModel(mem_bytes=mem * HW["kv_bytes"], page_size=16, **HW)
    oracle = OS.SchedulerOracle(OB.BuilderOracle(cm, [OB.Request(r.tokens, r.d_est, 0) for r in reqs]),
                                [r.d_true for r in reqs], mem, budget, pages)
    # inputs: weights, one x row per row slot of a step, an empty pool
    probe = W.assemble_batch(16, [(1, 1, -1)], 0, [], None)
    tens0 = W.make_tensors(shape, probe, seed, gains="random")
    rng = np.random.default_rng([seed, 9])
    x_all = W.round_to_bf16(rng.standard_normal((budget, shape.d_model), dtype=np.float32))
    kp = np.zeros((pages, 16, shape.n_kv_heads, shape.head_dim))
    vp = np.zeros_like(kp)
    layer = lib.Layer(shape, device=0)
    if flags:
        layer.set_overlap(head_cus_min=8, head_cus_max=16, tail_workgroups=8, min_prefill_rows=1, always=1)
    weights, keep = layer.upload_weights(tens0)
    dev = lib.binding_device_state(weights, keep, torch.from_numpy(x_all).cuda().to(torch.bfloat16),
                                   layer.pack_pool(W.f32_to_bf16_bits(kp.astype(np.float32)), W.f32_to_bf16_bits(vp.astype(np.float32))), pages)
    steps = 0
    while True:
        d, want = sched.next_step(), oracle.next_step()
        if want is None:
            assert d is None
            break
        for k in want:
            assert np.array_equal(np.asarray(want[k]), np.asarray(d[k])), (steps, k)
        batch = W.Batch(page_size=16, **{k: v for k, v in d.items() if k != "seq_request"})
        n = batch.n_rows
        tens = dataclasses.replace(tens0, x=x_all[:n], k_pool=kp, v_pool=vp)
        ref = O.layer_step(shape, tens, batch)
        diag = O.layer_step(shape, tens, batch, storage="bf16")
        dev_step = dataclasses.replace(dev, x=dev.x[:n])
        y = layer.blend_step(dev_step, batch, flags=flags)
        torch.cuda.synchronize()
        check(y.float().cpu().numpy().astype(np.float64), ref["y"], diag["y"], "pool seed %d step %d (%d rows)" % (seed, steps, n))
        # the oracle's pool after the step, stored as the pool stores it: in bfloat16
        kp, vp = O.append_kv(batch, ref, kp, vp)
        kp = W.round_to_bf16(kp.astype(np.float32)).astype(np.float64)
        vp = W.round_to_bf16(vp.astype(np.float32)).astype(np.float64)
        steps += 1
    assert steps == sched.stats()["steps"] and sched.stats()["finished"] == len(reqs)
    # the pools agree wherever something was ever written (the rest is zero on both sides)
    k, v = layer.unpack_pool(dev.kv_pool, pages)
    k, v = k.float().cpu().numpy().astype(np.float64), v.float().cpu().numpy().astype(np.float64)
    assert np.max(np.abs(k - kp)) <= 2e-2 * np.max(np.abs(kp)) and np.max(np.abs(v - vp)) <= 2e-2 * np.max(np.abs(vp))
    assert np.array_equal(k == 0, kp == 0) and np.array_equal(v == 0, vp == 0)


@pytest.mark.parametrize("policy", ["blend", "dfs", "random"])
def test_small_pool_runs_to_completion(lib, policy):
    reqs = W.synthetic_pool(5, n_groups=6, per_group=4, n_fresh=12)
    for r in reqs:                      # keep the run short
        r.d_true = min(r.d_true, 60)
        r.d_est = min(r.d_est, 60)
    shape = W.TINY
    mem = 30_000
    hw = dict(p_model=8_030_000_000, kv_bytes=shape.kv_bytes_per_token, compute=2.5e15, bandwidth=8e12)
    pages = mem // 16 * 2 + 4096
    b, s, _ = E.make_scheduler(lib, reqs, hw, mem, 512, pages, policy=policy, split_t=2048 if policy == "blend" else 0, split_budget=500)
    stepper = E.GpuStepper(lib, shape, 512, pages, seed=1)
    st = E.serve(s, stepper)
    ms = stepper.total_ms()
    assert st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
    assert len(stepper.events) == st["steps"] and ms > 0.0
    import torch
    assert bool(torch.isfinite(stepper.y[: 16].float()).all())
