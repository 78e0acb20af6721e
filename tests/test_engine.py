"""A pool served to completion through the library's scheduler, on the CPU: token and memory accounts
add up, every step is a descriptor the library accepts, and sharing is found by the orders that keep
a group's members together.  (Step-by-step parity with the oracle: tests/test_scheduler.py.)"""
import numpy as np
import pytest

from paper_2411_16102_amd import binding, engine as E, workloads as W

HW = dict(p_model=8_030_000_000, kv_bytes=1024 * 32 * 2 * 2, compute=2.5e15, bandwidth=8.0e12)


@pytest.mark.parametrize("policy", ["blend", "dfs", "random"])
@pytest.mark.parametrize("seed", [0, 1])
def test_pool_is_served_to_completion(policy, seed):
    reqs = W.synthetic_pool(seed, n_groups=6, per_group=5, n_fresh=10, templates="shuffled" if seed else "by_kind")
    mem, budget, pages = 60_000, 1024, 60_000 // 16 + 2048
    b, s, _ = E.make_scheduler(binding.load(), reqs, HW, mem, budget, pages, policy=policy, seed=seed,
                               split_t=10 ** 9 if policy == "blend" else 0, split_budget=2000)
    lay = binding.Layer(W.TINY, device=-1)
    seen = dict(rows=0, steps=0)

    def step(d):
        batch = W.Batch(page_size=16, **{k: v for k, v in d.items() if k != "seq_request"})
        assert lay.validate(batch) == 0, lay.last_error()
        assert 0 < d["n_rows"] <= budget
        seen["rows"] += d["n_rows"]
        seen["steps"] += 1

    st = E.serve(s, step)
    assert st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
    # every prompt token was either computed in a prefill row or skipped because a sharer had computed it
    assert st["prefill_rows"] + st["prompt_tokens_skipped"] == sum(len(r.tokens) for r in reqs)
    assert st["rows"] == seen["rows"] == st["prefill_rows"] + st["decode_rows"] and st["steps"] == seen["steps"]
    assert st["decode_rows"] == st["tokens_out"] - len(reqs)      # the first token comes from the last prompt row
    assert st["peak_tokens"] <= mem + max(len(r.tokens) + r.d_true for r in reqs)
    assert st["peak_pages"] <= pages


def test_sharing_is_found_by_the_dfs_order_and_lost_by_a_random_one():
    # groups of 8 behind a 600-token prefix, memory for about two groups: in DFS order the members
    # of a group are resident together and the prefix is computed once per group
    rng = np.random.default_rng(3)
    reqs = []
    for g in range(10):
        prefix = [int(t) for t in rng.integers(0, 1000, 600)]
        for _ in range(8):
            reqs.append(W.PoolRequest(prefix + [int(t) for t in rng.integers(0, 1000, 20)], 30, 30))
    reqs = [reqs[i] for i in rng.permutation(len(reqs))]
    skipped = {}
    for policy in ("dfs", "blend", "random"):
        _, s, _ = E.make_scheduler(binding.load(), reqs, HW, 2500, 512, 2500 // 16 + 512, policy=policy)
        skipped[policy] = E.serve(s, lambda d: None)["prompt_tokens_skipped"]
    whole_pages = (600 // 16) * 16        # what a sharer skips: the whole pages of the prefix
    # (a few tails happen to start with the same token and share a little more)
    assert 10 * 7 * whole_pages <= skipped["dfs"] < 10 * 7 * whole_pages + 20
    # Algorithm 1 only reorders siblings, so groups stay together; the one group in which the two
    # scanners meet may be served in two parts and compute its prefix twice
    assert skipped["dfs"] - 650 <= skipped["blend"] <= skipped["dfs"]
    assert skipped["random"] < skipped["dfs"]


def test_blend_fills_steps_that_the_dfs_order_leaves_to_decoding_alone():
    # compute-intensive requests (long prompts, short outputs) and memory-intensive ones (short prompts,
    # long outputs): the resource-aware order runs both kinds together, so fewer steps consist of a few
    # decode rows only; priced with a step cost that has a fixed part, that is a shorter run
    rng = np.random.default_rng(4)
    reqs = []
    # (the two kinds start with different tokens, as two datasets with their own templates would: the
    # prefix-DFS order then serves one kind after the other)
    for _ in range(240):
        reqs.append(W.PoolRequest([1] + [int(t) for t in rng.integers(0, 1000, int(rng.integers(600, 1200)))], 8, 8))
    for _ in range(30):
        reqs.append(W.PoolRequest([2] + [int(t) for t in rng.integers(0, 1000, int(rng.integers(20, 60)))], 400, 400))
    out = {}
    for policy in ("dfs", "blend"):
        _, s, _ = E.make_scheduler(binding.load(), reqs, HW, 24_000, 512, 24_000 // 16 + 1024, policy=policy)
        cost = [0.0]

        def step(d, cost=cost):
            cost[0] += 200.0 + d["n_rows"] * 0.4 + float(np.sum(d["kv_len"][d["n_prefill"]:])) * 0.001
        st = E.serve(s, step)
        out[policy] = (cost[0], st["steps"])
    print(out)
    assert out["blend"][1] < 0.75 * out["dfs"][1] and out["blend"][0] < out["dfs"][0]


def test_pool_is_served_under_the_shared_memory_model():
    reqs = W.synthetic_pool(3, n_groups=6, per_group=5, n_fresh=10)
    b, s, split = E.make_scheduler(binding.load(), reqs, HW, 60_000, 1024, 60_000 // 16 + 2048, policy="blend",
                                   split_t=10 ** 9, mem_model="shared")
    assert split is None                              # node splitting is switched off with this model
    st = E.serve(s, lambda d: None)
    assert st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
    assert st["prefill_rows"] + st["prompt_tokens_skipped"] == sum(len(r.tokens) for r in reqs)
    # groups look less memory-bound than under the paper's model, fresh prompts look the same
    ref, _, _ = E.make_scheduler(binding.load(), reqs, HW, 60_000, 1024, 60_000 // 16 + 2048, policy="blend")
    t_s, t_e = b.tree(), ref.tree()
    assert int(t_s["B"][0]) < int(t_e["B"][0]) and int(t_s["A"][0]) == int(t_e["A"][0])


def test_a_severely_underestimated_request_moves_to_the_memory_side():
    # prompt-heavy requests with short estimated outputs sit at the compute-intensive end; a few of
    # them decode eight times longer than estimated.  With relocation their reservations move to
    # the right partition once they have produced twice their estimate; the accounts still close.
    rng = np.random.default_rng(11)
    reqs = []
    for i in range(40):
        reqs.append(W.PoolRequest([int(t) for t in rng.integers(0, 1000, 300)], 8, 64 if i % 5 == 0 else 8))
    for i in range(40):
        reqs.append(W.PoolRequest([int(t) for t in rng.integers(0, 1000, 20)], 200, 200))
    stats = {}
    for pct in (200, 0):
        _, s, _ = E.make_scheduler(binding.load(), reqs, HW, 6000, 512, 6000 // 16 + 512, policy="blend", relocate_pct=pct)
        st = E.serve(s, lambda d: None)
        assert st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
        stats[pct] = (st["relocated"], st["steps"])
    assert stats[0][0] == 0
    assert 0 < stats[200][0] <= 8          # only the eight long decoders can move, and only those admitted on the left


def test_steps_with_prefill_rows_come_in_multiples_of_128():
    reqs = W.synthetic_pool(2, n_groups=6, per_group=5, n_fresh=30)
    rows = {}
    for mult in (128, 1):
        _, s, _ = E.make_scheduler(binding.load(), reqs, HW, 30_000, 1024, 30_000 // 16 + 2048, policy="blend", row_multiple=mult)
        seen = []
        st = E.serve(s, lambda d, seen=seen: seen.append((d["n_rows"], int(d["row_start"][d["n_prefill"]]))))
        assert st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
        assert st["prefill_rows"] + st["prompt_tokens_skipped"] == sum(len(r.tokens) for r in reqs)
        rows[mult] = seen
    # a step of more than 128 rows keeps a ragged row count only when it has no prefill rows left to give up
    assert all(n <= 128 or n % 128 == 0 or pf == 0 for n, pf in rows[128])
    assert any(n > 128 and n % 128 and pf for n, pf in rows[1])


def test_early_finish_and_overrun_keep_the_account_consistent():
    # outputs twice and half the estimates: reservations grow token by token or are returned early,
    # and a request admitted from the left that reaches twice its estimate moves to the right partition
    rng = np.random.default_rng(5)
    reqs = [W.PoolRequest([int(t) for t in rng.integers(0, 1000, int(rng.integers(20, 200)))], 0, 0) for _ in range(60)]
    for i, r in enumerate(reqs):
        r.d_est = int(rng.integers(4, 40))
        r.d_true = max(1, r.d_est * 3 if i % 3 == 0 else r.d_est // 2 if i % 3 == 1 else r.d_est)
    _, s, _ = E.make_scheduler(binding.load(), reqs, HW, 3000, 256, 3000 // 16 + 256, policy="blend")
    st = E.serve(s, lambda d: None)
    assert st["finished"] == 60 and st["tokens_out"] == sum(r.d_true for r in reqs)
    assert st["relocated"] >= 1
    _, s0, _ = E.make_scheduler(binding.load(), reqs, HW, 3000, 256, 3000 // 16 + 256, policy="blend", relocate_pct=0)
    assert E.serve(s0, lambda d: None)["relocated"] == 0
