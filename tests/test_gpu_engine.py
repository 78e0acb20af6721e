"""The multi-step driver on the GPU: a small pool served to completion through bs_blend_step
under each admission order; every step is accepted by the library and takes device time."""
import pytest

from paper_2411_16102_amd import engine as E, workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("policy", ["blend", "dfs", "random"])
def test_small_pool_runs_to_completion(lib, policy):
    reqs = E.synthetic_pool(5, n_groups=6, per_group=4, n_fresh=12)
    for r in reqs:                      # keep the run short
        r.d_true = min(r.d_true, 60)
        r.d_est = min(r.d_est, 60)
    shape = W.TINY
    mem = 30_000
    b = lib.Builder(8_030_000_000, shape.kv_bytes_per_token, 2.5e15, 8e12, mem * shape.kv_bytes_per_token, 16)
    eng = E.Engine(b, reqs, mem, policy=policy, token_budget=512, split_t=2048 if policy == "blend" else 0, split_budget=500)
    stepper = E.GpuStepper(lib, shape, 512, mem // 16 * 2 + 4096, seed=1)
    st = eng.run(stepper)
    ms = stepper.total_ms()
    assert eng.done and st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
    assert len(stepper.events) == st["steps"] and ms > 0.0
    import torch
    assert bool(torch.isfinite(stepper.y[: 16].float()).all())
