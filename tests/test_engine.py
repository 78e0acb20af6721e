"""The multi-step driver on the CPU: every request is served to completion, token and memory
accounts add up, every emitted step is a descriptor the library accepts, and shared prompt
segments are computed once while their sharers overlap in time.  Steps are priced by a linear
cost function instead of being run (the GPU run is in test_gpu_parity.py)."""
import numpy as np
import pytest

from paper_2411_16102_amd import binding, engine as E, workloads as W

HW = dict(p_model=8_030_000_000, kv_bytes=1024 * 32 * 2 * 2, compute=2.5e15, bandwidth=8.0e12)


def make_engine(reqs, policy, mem_tokens=60_000, budget=1024, **kw):
    b = binding.Builder(HW["p_model"], HW["kv_bytes"], HW["compute"], HW["bandwidth"], mem_tokens * HW["kv_bytes"], 16)
    return E.Engine(b, reqs, mem_tokens, policy=policy, token_budget=budget, **kw)


@pytest.mark.parametrize("policy", ["blend", "dfs", "random"])
@pytest.mark.parametrize("seed", [0, 1])
def test_pool_is_served_to_completion(policy, seed):
    reqs = E.synthetic_pool(seed, n_groups=6, per_group=5, n_fresh=10)
    eng = make_engine(reqs, policy, split_t=10 ** 9 if policy == "blend" else 0, split_budget=2000)
    lay = binding.Layer(W.TINY, device=-1)
    seen = dict(rows=0, steps=0, max_rows=0)

    def step(d):
        batch = W.Batch(page_size=16, **{k: v for k, v in d.items() if k != "seq_request"})
        assert lay.validate(batch) == 0, lay.last_error()
        assert 0 < d["n_rows"] <= eng.token_budget
        seen["rows"] += d["n_rows"]
        seen["steps"] += 1
        seen["max_rows"] = max(seen["max_rows"], d["n_rows"])

    st = eng.run(step)
    assert eng.done and st["finished"] == len(reqs)
    assert st["tokens_out"] == sum(r.d_true for r in reqs)
    # every prompt token was either computed in a prefill row or skipped because a sharer had computed it
    assert st["prefill_rows"] + st["prompt_tokens_skipped"] == sum(len(r.tokens) for r in reqs)
    assert st["rows"] == seen["rows"] == st["prefill_rows"] + st["decode_rows"] and st["steps"] == seen["steps"]
    assert st["decode_rows"] == st["tokens_out"] - len(reqs)      # the first token comes from the last prompt row
    assert eng.used == [0, 0] and not eng.node_ref.any()
    assert st["peak_tokens"] <= eng.mem_tokens + max(len(r.tokens) + r.d_true for r in reqs)


def test_sharing_is_found_by_the_dfs_order_and_lost_by_a_random_one():
    # groups of 8 behind a 600-token prefix, memory for about two groups: in DFS order the members
    # of a group are resident together and the prefix is computed once per group
    rng = np.random.default_rng(3)
    reqs = []
    for g in range(10):
        prefix = [int(t) for t in rng.integers(0, 1000, 600)]
        for _ in range(8):
            reqs.append(E.PoolRequest(prefix + [int(t) for t in rng.integers(0, 1000, 20)], 30, 30))
    perm = rng.permutation(len(reqs))
    reqs = [reqs[i] for i in perm]
    skipped = {}
    for policy in ("dfs", "blend", "random"):
        eng = make_engine(reqs, policy, mem_tokens=2500, budget=512)
        skipped[policy] = eng.run(lambda d: None)["prompt_tokens_skipped"]
    # (a few tails happen to start with the same token and share a little more)
    assert 10 * 7 * 600 <= skipped["dfs"] < 10 * 7 * 600 + 20
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
        reqs.append(E.PoolRequest([1] + [int(t) for t in rng.integers(0, 1000, int(rng.integers(600, 1200)))], 8, 8))
    for _ in range(30):
        reqs.append(E.PoolRequest([2] + [int(t) for t in rng.integers(0, 1000, int(rng.integers(20, 60)))], 400, 400))
    out = {}
    for policy in ("dfs", "blend"):
        eng = make_engine(reqs, policy, mem_tokens=24_000, budget=512)
        cost = [0.0]

        def step(d, cost=cost):
            cost[0] += 200.0 + d["n_rows"] * 0.4 + float(np.sum(d["kv_len"][d["n_prefill"]:])) * 0.001
        st = eng.run(step)
        out[policy] = (cost[0], st["steps"])
    print(out)
    assert out["blend"][1] < 0.75 * out["dfs"][1] and out["blend"][0] < out["dfs"][0]


def test_pool_is_served_under_the_shared_memory_model():
    reqs = E.synthetic_pool(3, n_groups=6, per_group=5, n_fresh=10)
    eng = make_engine(reqs, "blend", split_t=10 ** 9, mem_model="shared")
    assert eng.split_info is None                     # node splitting is switched off with this model
    st = eng.run(lambda d: None)
    assert eng.done and st["finished"] == len(reqs)
    assert st["tokens_out"] == sum(r.d_true for r in reqs)
    assert st["prefill_rows"] + st["prompt_tokens_skipped"] == sum(len(r.tokens) for r in reqs)
    # groups look less memory-bound than under the paper's model, fresh prompts look the same
    ref = make_engine(reqs, "blend")
    t_s, t_e = eng.b.tree(), ref.b.tree()
    assert int(t_s["B"][0]) < int(t_e["B"][0]) and int(t_s["A"][0]) == int(t_e["A"][0])


def test_a_severely_underestimated_request_moves_to_the_memory_side():
    # prompt-heavy requests with short estimated outputs sit at the compute-intensive end; a few of
    # them decode eight times longer than estimated.  With relocation their reservations move to
    # the right partition once they have produced twice their estimate; the accounts still close.
    rng = np.random.default_rng(11)
    reqs = []
    for i in range(40):
        reqs.append(E.PoolRequest([int(t) for t in rng.integers(0, 1000, 300)], 8, 64 if i % 5 == 0 else 8))
    for i in range(40):
        reqs.append(E.PoolRequest([int(t) for t in rng.integers(0, 1000, 20)], 200, 200))
    stats = {}
    for factor in (2.0, 0.0):
        eng = make_engine(reqs, "blend", mem_tokens=6000, budget=512, relocate_factor=factor)
        peak_left = [0]

        def step(d, eng=eng, peak_left=peak_left):
            peak_left[0] = max(peak_left[0], eng.used[0])

        st = eng.run(step)
        assert eng.done and st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
        assert eng.used == [0, 0] and not eng.node_ref.any()
        stats[factor] = (st["relocated"], st["steps"])
    assert stats[0.0][0] == 0
    assert 0 < stats[2.0][0] <= 8          # only the eight long decoders can move, and only those admitted on the left


def test_steps_with_prefill_rows_come_in_multiples_of_128():
    reqs = E.synthetic_pool(2, n_groups=6, per_group=5, n_fresh=30)
    rows = {}
    for mult in (128, 1):
        eng = make_engine(reqs, "blend", mem_tokens=30_000, budget=1024, row_multiple=mult)
        seen = []
        st = eng.run(lambda d, seen=seen: seen.append((d["n_rows"], int(d["row_start"][d["n_prefill"]]))))
        assert eng.done and st["finished"] == len(reqs) and st["tokens_out"] == sum(r.d_true for r in reqs)
        assert st["prefill_rows"] + st["prompt_tokens_skipped"] == sum(len(r.tokens) for r in reqs)
        rows[mult] = seen
    # a step of more than 128 rows keeps a ragged row count only when it has no prefill rows left to give up
    assert all(n <= 128 or n % 128 == 0 or pf == 0 for n, pf in rows[128])
    assert any(n > 128 and n % 128 and pf for n, pf in rows[1])
