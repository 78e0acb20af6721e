"""Pins for the batch-builder oracle: the paper's printed example, its algebraic
identities, and brute force on small random request pools."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import builder as B
from paper_2411_16102_amd import workloads as W


def read_golden(name):
    vals = {}
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


A100 = dict(compute=312e12, bandwidth=2.039e12)
LLAMA8B = dict(p_model=8_030_000_000, kv_bytes=1024 * 32 * 4)   # H_kv * L * 4 with H_kv = 8 * 128, L = 32


def cm(**kw):
    d = dict(p_model=LLAMA8B["p_model"], kv_bytes=LLAMA8B["kv_bytes"], compute=A100["compute"],
             bandwidth=A100["bandwidth"], mem_bytes=60 * 10 ** 9, page_size=16)
    d.update(kw)
    return B.CostModel(**d)


# ---------------------------------------------------------------------------
# the paper's printed values and identities
# ---------------------------------------------------------------------------
def test_memory_partition_example_of_figure_6():
    g = read_golden("fig6_memory_partition.txt")
    m_l, m_r = B.memory_partition(g["rho_root"], g["rho_left"], g["rho_right"], g["memory_gb"])
    assert abs(m_l - g["m_left_gb"]) <= 0.1 and abs(m_r - g["m_right_gb"]) <= 0.1
    # both constraints of Section 5.3 hold for the computed split
    assert abs(m_l + m_r - g["memory_gb"]) < 1e-12
    assert abs(m_l * g["rho_left"] + m_r * g["rho_right"] - g["memory_gb"] * g["rho_root"]) < 1e-9
    # and the printed identity holds for the printed, rounded values
    assert abs(g["rho_left"] * g["m_left_gb"] + g["rho_right"] * g["m_right_gb"] - g["rho_root"] * g["memory_gb"]) < 0.5  # 75.9 vs 76.2: printed to 3 digits


def test_memory_partition_degenerate_cases():
    assert B.memory_partition(1.0, 2.0, 2.0, 10.0) == (10.0, 0.0)       # equal densities
    assert B.memory_partition(5.0, 2.0, 1.0, 10.0) == (10.0, 0.0)       # target above the left density: clamp
    assert B.memory_partition(0.5, 2.0, 1.0, 10.0) == (0.0, 10.0)       # target below the right density
    assert B.memory_partition(1.0, float("inf"), 0.5, 10.0) == (0.0, 10.0)  # left side never decodes


@pytest.mark.parametrize("p,d", [(100, 50), (1024, 16), (7, 4000), (512, 512)])
def test_batch_density_equals_request_density(p, d):
    # Section 4.2: Comp(B)/Mem(B) with B_decode = KV-Mem / ((p + d/2) kappa) requests and a
    # prefill:decode token ratio of p/d equals the request-level density, for any KV-Mem
    c = cm()
    req = B.Request(tokens=list(range(p)), d_est=d)
    o = B.BuilderOracle(c, [req])
    leaf = [n for n in o.nodes if n.req == 0][0]
    rho_r = B.rho_value(c, leaf.A, leaf.B)
    kv_mem = Fraction(37 * 10 ** 9)
    b_decode = kv_mem / ((Fraction(p) + Fraction(d, 2)) * c.kv_bytes)
    comp_b = b_decode * Fraction(p + d, d) * c.p_model * 2 / Fraction(c.compute)
    mem_b = kv_mem / Fraction(c.bandwidth)
    assert abs(float(comp_b / mem_b) / rho_r - 1.0) < 1e-12
    # and the request-level form itself: 2 (p + d) P / compute over (p d + d^2/2) kappa / bandwidth
    direct = (2 * (p + d) * c.p_model / c.compute) / ((p * d + d * d / 2) * c.kv_bytes / c.bandwidth)
    assert abs(direct / rho_r - 1.0) < 1e-12


def test_memory_time_is_linear_in_loaded_tokens():
    # Table 1: attention estimates for 512 / 768 / 1024 sequences of context 1024 are in ratio 1 : 1.5 : 2.
    g = read_golden("table1_attention_estimates.txt")
    c = cm()
    t = []
    for n in (512, 768, 1024):
        # one decode step over n sequences of context 1024 = n requests with p = 1023, d = 1
        # loads sum (p + i) = 1024 tokens each
        reqs = [B.Request(tokens=[k] + list(range(1022)), d_est=1) for k in range(n)]
        o = B.BuilderOracle(c, reqs)
        t.append(o.nodes[0].B)            # proportional to T_mem
    assert t[1] * 2 == t[0] * 3 and t[2] == t[0] * 2
    assert abs(g["est_768"] / g["est_512"] - t[1] / t[0]) < 2e-3
    assert abs(g["est_1024"] / g["est_512"] - t[2] / t[0]) < 2e-3
    # B counts 2 p d + d^2 = 2 * (loaded tokens) - d: 2 * 1024 - 1 per sequence here
    assert t[0] == 512 * (2 * 1023 + 1)


# ---------------------------------------------------------------------------
# brute force on small pools
# ---------------------------------------------------------------------------
def random_pool(seed, n=8, vocab=3, max_len=7):
    rng = np.random.default_rng(seed)
    reqs = []
    for _ in range(n):
        L = int(rng.integers(1, max_len + 1))
        reqs.append(B.Request(tokens=[int(t) for t in rng.integers(0, vocab, L)], d_est=int(rng.integers(0, 9))))
    return reqs


def lcp(a, b):
    n = 0
    while n < min(len(a), len(b)) and a[n] == b[n]:
        n += 1
    return n


def subtree_requests(o, n):
    nd = o.nodes[n]
    if nd.req >= 0:
        return [nd.req]
    out = []
    for c in nd.children:
        out += subtree_requests(o, c)
    return out


@pytest.mark.parametrize("seed", range(12))
def test_trie_against_brute_force(seed):
    reqs = random_pool(seed)
    o = B.BuilderOracle(cm(), reqs)
    leaf_of = {nd.req: i for i, nd in enumerate(o.nodes) if nd.req >= 0}
    assert sorted(leaf_of) == list(range(len(reqs)))

    def ancestors(n):
        out = []
        while n >= 0:
            out.append(n)
            n = o.nodes[n].parent
        return out
    # the deepest common internal node of two requests ends exactly at their common prefix length
    for a, b in itertools.combinations(range(len(reqs)), 2):
        anc_a = ancestors(o.nodes[leaf_of[a]].parent)
        anc_b = set(ancestors(o.nodes[leaf_of[b]].parent))
        lca = next(n for n in anc_a if n in anc_b)
        assert o.nodes[lca].end == lcp(reqs[a].tokens, reqs[b].tokens)
    # segments chain without gaps; every internal node (but the root) is a true branching point
    for i, nd in enumerate(o.nodes):
        if nd.parent >= 0:
            assert nd.start == o.nodes[nd.parent].end
        if nd.req < 0 and i != 0:
            assert len(nd.children) >= 2 and nd.end > nd.start
        if nd.req >= 0:
            assert nd.end == len(reqs[nd.req].tokens)
    # A = distinct prompt prefixes (= distinct tokens of the trie) in the subtree with the root
    # path counted once, + outputs;  B = sum 2 p d + d^2
    for i, nd in enumerate(o.nodes):
        rs = subtree_requests(o, i)
        prefixes = set()
        for r in rs:
            for k in range(1, len(reqs[r].tokens) + 1):
                prefixes.add(tuple(reqs[r].tokens[:k]))
        assert nd.A == len(prefixes) + sum(reqs[r].d_est for r in rs)
        assert nd.B == sum(2 * len(reqs[r].tokens) * reqs[r].d_est + reqs[r].d_est ** 2 for r in rs)


@pytest.mark.parametrize("seed", range(12))
def test_sort_keeps_the_trie_and_orders_siblings(seed):
    reqs = random_pool(seed, n=8)
    o = B.BuilderOracle(cm(), reqs)
    # same tree as an unsorted build: parent -> set of (child segment, requests below)
    def shape(o):
        return {(nd.start, nd.end, tuple(sorted(subtree_requests(o, i)))) for i, nd in enumerate(o.nodes)}
    class Unsorted(B.BuilderOracle):
        def _layer_sort(self, n):
            pass
    assert shape(o) == shape(Unsorted(cm(), reqs))
    # siblings: density non-increasing left to right, by exact rational comparison from the definition
    for nd in o.nodes:
        ds = []
        for c in nd.children:
            ch = o.nodes[c]
            ds.append(math.inf if ch.B == 0 else Fraction(ch.A, ch.B))
        assert all(ds[k] >= ds[k + 1] for k in range(len(ds) - 1))
    # every node's requests are contiguous in the leaf order (a DFS order keeps prefix sharing)
    t = o.tree_arrays()
    for i in range(len(t["parent"])):
        got = sorted(t["leaf_order"][t["first_leaf"][i]:t["first_leaf"][i] + t["leaf_count"][i]])
        nid = o.dfs[i]
        assert got == sorted(subtree_requests(o, nid))
    # parents precede children in the numbering
    assert all(t["parent"][i] < i for i in range(len(t["parent"])))


def test_ties_go_to_the_smaller_request_index():
    reqs = [B.Request([1, 5], 3), B.Request([2, 5], 3), B.Request([0, 5], 3)]
    o = B.BuilderOracle(cm(), reqs)
    assert list(o.leaf_order) == [0, 1, 2]


def test_compute_intensive_left_memory_intensive_right():
    # long prompt / short output is compute-intensive; short prompt / long output memory-intensive
    reqs = [B.Request([9] * 10 + [k], 4000) for k in range(3)] + [B.Request([7] * 900 + [k], 2) for k in range(3)]
    o = B.BuilderOracle(cm(), reqs)
    assert set(o.leaf_order[:3]) == {3, 4, 5} and set(o.leaf_order[3:]) == {0, 1, 2}


# ---------------------------------------------------------------------------
# dual scan and the emitted descriptor
# ---------------------------------------------------------------------------
def mixed_pool(seed, n_groups=3, per_group=5, n_fresh=6):
    rng = np.random.default_rng(seed)
    reqs = []
    for g in range(n_groups):
        prefix = [int(t) for t in rng.integers(0, 1000, int(rng.integers(20, 90)))]
        for _ in range(per_group):
            own = [int(t) for t in rng.integers(0, 1000, int(rng.integers(1, 30)))]
            toks = prefix + own
            reqs.append(B.Request(toks, d_est=int(rng.integers(50, 400)), n_cached=len(toks) + int(rng.integers(0, 60))))
    for _ in range(n_fresh):
        toks = [int(t) for t in rng.integers(0, 1000, int(rng.integers(40, 200)))]
        reqs.append(B.Request(toks, d_est=int(rng.integers(1, 20)), n_cached=0))
    return reqs


@pytest.mark.parametrize("seed", range(6))
def test_budgets_follow_algorithm_3(seed):
    reqs = mixed_pool(seed)
    c = cm(mem_bytes=3_000_000_000)
    o = B.BuilderOracle(c, reqs)
    b = o.budgets()
    M = float(c.mem_bytes)
    assert abs(b["m_l"] + b["m_r"] - M) < 1e-3
    if b["rho_l"] != b["rho_r"] and b["rho_r"] <= b["rho_rt"] <= b["rho_l"] and math.isfinite(b["rho_l"]):
        assert abs(b["m_l"] * b["rho_l"] + b["m_r"] * b["rho_r"] - M * b["rho_rt"]) <= 1e-6 * M * b["rho_rt"]
    rt, L, R = o.scan_sides()
    for tag, n in (("l", L), ("r", R)):
        nd = o.nodes[n]
        p_bar, d_bar = Fraction(nd.sum_p, nd.n_req), Fraction(nd.sum_d, nd.n_req)
        n_exact = Fraction(b["m_" + tag]) / ((p_bar + d_bar / 2) * c.kv_bytes)
        assert abs(b["n_" + tag] - max(1, math.floor(n_exact))) <= 1
        if d_bar:
            assert abs(b["c_" + tag] - math.floor(b["n_" + tag] * p_bar / d_bar)) <= 1


@pytest.mark.parametrize("seed", range(6))
def test_emitted_descriptor_is_consistent(seed):
    reqs = mixed_pool(seed)
    c = cm(mem_bytes=40_000_000)
    o = B.BuilderOracle(c, reqs)
    info, d = o.next_batch(prefill_budget=256)
    assert d["n_seq"] == info["n_prefill"] + info["n_decode"] and d["n_seq"] > 0
    ps = c.page_size
    # every request at most once; prefill chunks within budget and within the prompt
    assert len(set(d["seq_request"])) == d["n_seq"]
    q = np.diff(d["row_start"])
    assert q[:d["n_prefill"]].sum() <= 256
    for s in range(d["n_seq"]):
        r = reqs[d["seq_request"][s]]
        if s < d["n_prefill"]:
            assert r.n_cached < len(r.tokens) and d["kv_len"][s] == r.n_cached + q[s] <= len(r.tokens)
        else:
            assert r.n_cached >= len(r.tokens) and q[s] == 1 and d["kv_len"][s] == r.n_cached + 1
        assert d["page_start"][s + 1] - d["page_start"][s] == -(-d["kv_len"][s] // ps)
    # decode sequences follow the leaf order; each node's members are a contiguous run whose
    # prompts agree on every token of the node's pages; shared pages appear once physically
    pos = {ri: k for k, ri in enumerate(o.leaf_order)}
    dec = list(d["seq_request"][d["n_prefill"]:])
    assert dec == sorted(dec, key=lambda ri: pos[ri])
    used = {}
    for n in range(d["n_nodes"]):
        f, cnt = d["node_seq_first"][n], d["node_seq_count"][n]
        assert cnt >= 2
        pages = d["node_page_ids"][d["node_page_start"][n]:d["node_page_start"][n + 1]]
        assert len(pages) >= 1
        depth = 0
        k = n
        while d["node_parent"][k] >= 0:
            k = d["node_parent"][k]
            depth += d["node_page_start"][k + 1] - d["node_page_start"][k]
        toks = None
        for s in range(f, f + cnt):
            tab = d["page_ids"][d["page_start"][s] + depth:d["page_start"][s] + depth + len(pages)]
            assert list(tab) == list(pages)
            mine = reqs[d["seq_request"][s]].tokens[:(depth + len(pages)) * ps]
            assert len(mine) == (depth + len(pages)) * ps
            toks = mine if toks is None else toks
            assert mine == toks
        for p in pages:
            assert p not in used
            used[p] = n
    # private pages are private
    flat = list(d["page_ids"])
    for p in set(flat):
        if p not in used:
            assert flat.count(p) == 1
    assert max(flat) < d["n_pages"]
    # the GPU library's own validator accepts it
    from paper_2411_16102_amd import binding
    lay = binding.Layer(W.TINY, device=-1)
    batch = W.Batch(page_size=ps, n_seq=d["n_seq"], n_prefill=d["n_prefill"], n_rows=d["n_rows"],
                    row_start=d["row_start"], kv_len=d["kv_len"], page_start=d["page_start"], page_ids=d["page_ids"],
                    n_nodes=d["n_nodes"], node_parent=d["node_parent"], node_page_start=d["node_page_start"],
                    node_page_ids=d["node_page_ids"], node_seq_first=d["node_seq_first"],
                    node_seq_count=d["node_seq_count"], seq_leaf_node=d["seq_leaf_node"], n_pages=d["n_pages"])
    assert lay.validate(batch) == 0, lay.last_error()


def test_scanners_take_from_both_ends():
    # compute-heavy fresh prompts on the left, memory-heavy decoders on the right: a step holds both
    reqs = [B.Request([1000 + k] + [5] * 300, d_est=4, n_cached=0) for k in range(6)]
    reqs += [B.Request([2000 + k] + [6] * 20, d_est=3000, n_cached=21 + 500) for k in range(40)]
    o = B.BuilderOracle(cm(mem_bytes=200_000_000), reqs)
    info, d = o.next_batch()
    assert info["n_prefill"] >= 1 and info["n_decode"] >= 1
    assert info["rho_l"] > info["rho_rt"] > info["rho_r"]
    assert 0 < info["m_l"] < 200_000_000


# ---------------------------------------------------------------------------
# conditional node splitting (Section 5.2, Algorithm 2; Section 5.4, stopping conditions)
# ---------------------------------------------------------------------------
def leaf_density(o):
    return [None if b == 0 else Fraction(a, b) for a, b in o.leaf_keys()]


def non_increasing(fr):
    big = Fraction(10 ** 30)
    v = [big if f is None else f for f in fr]
    return all(v[i] >= v[i + 1] for i in range(len(v) - 1))


def brute_force_longest_non_increasing(vals):
    best = 0
    n = len(vals)
    for mask in range(1 << n):
        pick = [vals[i] for i in range(n) if mask >> i & 1]
        if all(pick[i] >= pick[i + 1] for i in range(len(pick) - 1)):
            best = max(best, len(pick))
    return best


@pytest.mark.parametrize("seed", range(20))
def test_longest_non_increasing_against_brute_force(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 11))
    keys = [(int(rng.integers(1, 6)), int(rng.integers(0, 5))) for _ in range(n)]   # B = 0 is +infinity
    got = B.longest_non_increasing(keys)
    vals = [Fraction(10 ** 9) if b == 0 else Fraction(a, b) for a, b in keys]
    assert got == sorted(got) and len(set(got)) == len(got)
    assert all(vals[got[i]] >= vals[got[i + 1]] for i in range(len(got) - 1))
    assert len(got) == brute_force_longest_non_increasing(vals)


def distinct_tokens(o):
    return o.nodes[0].A - sum(int(r.d_est) for r in o.reqs)


@pytest.mark.parametrize("seed", range(8))
def test_split_bounds_and_invariants(seed):
    reqs = mixed_pool(seed, n_groups=4, per_group=6, n_fresh=5)
    base = B.BuilderOracle(cm(), reqs)
    # t = 0: nothing shares zero tokens and sits below an internal node, so nothing moves
    o0 = B.BuilderOracle(cm(), reqs)
    assert o0.split(0) == dict(n_split=0, rounds=0, recompute_tokens=0, monotone=non_increasing(leaf_density(base)))
    assert o0.leaf_order == base.leaf_order
    # unlimited threshold: ends with a non-increasing leaf order (C1), every leaf moved at most once
    o = B.BuilderOracle(cm(), reqs)
    info = o.split(10 ** 9)
    assert info["monotone"] and non_increasing(leaf_density(o))
    assert info["n_split"] == len(o.detached) <= len(reqs)
    assert 0 < info["rounds"] <= info["n_split"] or info["n_split"] == 0
    for r in o.detached:                      # relocated leaves hang under the root with their whole prompt
        nd = [n for n in o.nodes if n.req == r][0]
        assert nd.parent == 0 and nd.start == 0 and nd.end == len(reqs[r].tokens)
    # sharing lost is at most the recomputed tokens, and nothing else changed: same requests, same B
    assert 0 <= distinct_tokens(o) - distinct_tokens(base) <= info["recompute_tokens"]
    assert sorted(o.leaf_order) == list(range(len(reqs))) and o.nodes[0].B == base.nodes[0].B
    # a finite threshold and a budget are both respected; relocated leaves are a subset of movable ones
    for t, budget in ((30, -1), (10 ** 9, 120), (45, 60)):
        ot = B.BuilderOracle(cm(), reqs)
        it = ot.split(t, budget)
        assert it["recompute_tokens"] <= (budget if budget >= 0 else 10 ** 18)
        for r in ot.detached:
            leaf = [n for n in base.nodes if n.req == r][0]
            assert leaf.parent != 0 and leaf.start <= t or r in o.detached
        if it["n_split"] == 0:
            assert ot.leaf_order == base.leaf_order


def test_split_separates_the_low_density_request_of_the_overview_figure():
    # Figure 3 (design overview), step 3, and Section 5.2: a request of low compute density that
    # shares its prefix with compute-intensive requests is separated from them and placed at the
    # memory-intensive end, its prefix recomputed.  Requests 0 and 1 (short outputs) share a
    # prefix with request 2 (long output); two memory-intensive requests without sharing follow.
    # rho of a node is sum A / sum B, so request 2 drags its whole group behind them: before the
    # split the compute-intensive requests 0 and 1 sit in the right half of the order.
    P = list(range(100, 140))
    Q = list(range(200, 220))
    reqs = [B.Request(P + Q + [1, 2, 3], d_est=4),        # compute-intensive
            B.Request(P + [7, 8, 9, 10], d_est=4),        # compute-intensive
            B.Request(P + Q + [4, 5, 6], d_est=10000),    # the outlier
            B.Request([50 + i for i in range(30)], d_est=400),
            B.Request([90 - i for i in range(30)], d_est=300)]
    o = B.BuilderOracle(cm(), reqs)
    assert not non_increasing(leaf_density(o))
    assert set(o.leaf_order[:2]) == {3, 4} and o.leaf_order[-1] == 2
    info = o.split(t=len(P) + len(Q))
    assert info == dict(n_split=1, rounds=1, recompute_tokens=len(P) + len(Q), monotone=True)
    assert o.detached == {2} and o.leaf_order[-1] == 2 and set(o.leaf_order[:2]) == {0, 1}
    # requests 0 and 1 still share their prefix: only the relocated request lost it
    assert distinct_tokens(o) - distinct_tokens(B.BuilderOracle(cm(), reqs)) == len(P) + len(Q)
    # with a threshold below its shared prefix the request cannot move (C2): the cheaper of the
    # compute-intensive requests goes instead, the other one stays out of order
    o2 = B.BuilderOracle(cm(), reqs)
    i2 = o2.split(t=len(P) + len(Q) - 1)
    assert 2 not in o2.detached and not i2["monotone"]


# ---------------------------------------------------------------------------
# memory model with prefix pages read once, and kappa of the attention variants
# ---------------------------------------------------------------------------
def loaded_tokens_when_decoding_together(reqs, members):
    """Section 4.1's count of loaded tokens, sum over decode steps i of (p + i) per request,
    taken literally step by step for `members` decoding together, but with every distinct
    prompt position (a position in the trie = a distinct prompt prefix) loaded once per step."""
    total = 0
    for i in range(1, max([reqs[r].d_est for r in members] + [0]) + 1):
        active = [r for r in members if reqs[r].d_est >= i]
        prefixes = {tuple(reqs[r].tokens[:k]) for r in active for k in range(1, len(reqs[r].tokens) + 1)}
        total += len(prefixes) + i * len(active)
    return total


@pytest.mark.parametrize("seed", range(12))
def test_shared_memory_model_against_step_by_step_count(seed):
    reqs = random_pool(seed, n=9)
    o = B.BuilderOracle(cm(mem_model="shared"), reqs)
    e = B.BuilderOracle(cm(), reqs)
    for n, nd in enumerate(o.nodes):
        members = subtree_requests(o, n)
        # the closed form drops the same d/2 per request as the paper's (p d + d^2 / 2)
        want = 2 * loaded_tokens_when_decoding_together(reqs, members) - sum(reqs[r].d_est for r in members)
        assert nd.B == want, (n, nd.B, want)
    # A does not depend on the memory model; B never exceeds the paper's
    key = lambda t: sorted((nd.start, nd.end, nd.req, nd.A) for nd in t.nodes)
    assert key(o) == key(e)
    assert o.nodes[0].B <= e.nodes[0].B


def test_shared_memory_model_equals_the_papers_without_sharing():
    reqs = [B.Request(tokens=[i] + [7] * (3 + i), d_est=2 * i + 1) for i in range(6)]   # distinct first tokens
    o = B.BuilderOracle(cm(mem_model="shared"), reqs)
    e = B.BuilderOracle(cm(), reqs)
    assert o.tree_arrays()["B"].tolist() == e.tree_arrays()["B"].tolist()
    assert o.leaf_order == e.leaf_order


def test_shared_memory_model_closed_form_for_one_group():
    # n requests behind one prefix of P tokens, each with o own tokens and the same d:
    # the prefix is read d times in all instead of n d times
    n, P, own, d = 5, 40, 3, 11
    reqs = [B.Request(tokens=[1] * P + [10 + i] * own, d_est=d) for i in range(n)]
    o = B.BuilderOracle(cm(mem_model="shared"), reqs)
    e = B.BuilderOracle(cm(), reqs)
    assert e.nodes[0].B == n * (2 * (P + own) * d + d * d)
    assert o.nodes[0].B == 2 * P * d + n * (2 * own * d + d * d)
    with pytest.raises(ValueError):
        o.split(100)


def test_kv_bytes_of_the_attention_variants():
    # Llama-3-8B, GQA with 8 KV heads of 128, 32 layers, 2-byte elements: H_kv * L * 4 with H_kv = 1024
    assert B.kv_bytes_per_token("gqa", 32, 32, 128, n_kv_heads=8) == 1024 * 32 * 4 == LLAMA8B["kv_bytes"]
    mha = B.kv_bytes_per_token("mha", 32, 32, 128)
    assert mha == 4096 * 32 * 4                                   # H_kv = H for multi-head attention
    assert B.kv_bytes_per_token("gqa", 32, 32, 128, n_kv_heads=32) == mha
    assert B.kv_bytes_per_token("mqa", 32, 32, 128) == mha // 32 == B.kv_bytes_per_token("gqa", 32, 32, 128, n_kv_heads=1)
    # a latent of 512 plus a rotary key of 64 per token and layer, 60 layers
    assert B.kv_bytes_per_token("mla", 60, 128, 128, latent_dim=512, rope_dim=64) == 576 * 60 * 2
    assert B.kv_bytes_per_token("gqa", 32, 32, 128, n_kv_heads=8, elem_bytes=1) == 1024 * 32 * 2
    for bad in (dict(variant="gqa", n_layers=32, n_heads=32, head_dim=128, n_kv_heads=5),
                dict(variant="mla", n_layers=60, n_heads=128, head_dim=128),
                dict(variant="xyz", n_layers=1, n_heads=1, head_dim=1)):
        with pytest.raises(ValueError):
            B.kv_bytes_per_token(**bad)


# ---------------------------------------------------------------------------
# hand-worked pins of the admission (Algorithm 3, Section 5.3), of the descriptor numbering and of
# the stopping conditions of node splitting (Section 5.4)
# ---------------------------------------------------------------------------
def unit_cost_model(mem_bytes):
    # 2 P / compute = 1/2 and kappa / (2 bandwidth) = 1/2, so rho(R) = A / B; kappa = 1 byte per token
    return B.CostModel(p_model=1, kv_bytes=1, compute=4.0, bandwidth=1.0, mem_bytes=mem_bytes, page_size=16)


def hand_pool():
    """Six requests.  0, 1, 2: prompts still to be prefilled, short outputs (compute-intensive);
    3 and 4 decode and share a 20-token prefix; 5 decodes a long output (memory-intensive)."""
    return [B.Request([1] * 40, d_est=10, n_cached=0),
            B.Request([2] * 30, d_est=10, n_cached=0),
            B.Request([3] * 20, d_est=20, n_cached=0),
            B.Request([4] * 20 + [5] * 4, d_est=40, n_cached=33),
            B.Request([4] * 20 + [6] * 12, d_est=40, n_cached=35),
            B.Request([7] * 10, d_est=100, n_cached=40)]


def test_next_batch_admits_what_algorithm_3_says_on_a_hand_worked_pool():
    # Densities by hand, rho(r) = (p + d) / (2 p d + d^2) (Section 4.1 without the p^2 term):
    #   r0 50/900   r1 40/700   r2 40/1200   r3 64/3520   r4 72/4160   r5 110/12000
    #   group G = {r3, r4}: A = 20 + 4 + 12 distinct prompt tokens + 80 outputs = 116, B = 7680
    # Root children by density, compute-intensive first: r1, r0, r2, G (r3 before r4), r5.
    o = B.BuilderOracle(unit_cost_model(1000), hand_pool())
    assert o.leaf_order == [1, 0, 2, 3, 4, 5]
    # Algorithm 3 with R_L = r1, R_R = r5 and the root: A = 136 + 220 = 356, B = 22480
    rho_rt, rho_l, rho_r = Fraction(356, 22480), Fraction(40, 700), Fraction(110, 12000)
    M = 1000
    m_l = M * (rho_rt - rho_r) / (rho_l - rho_r)
    m_r = M - m_l
    assert 139 < m_l < 140                                   # 139.02 by hand
    n_l = math.floor(m_l / (30 + Fraction(10, 2)))           # N = M_X / ((p + d/2) kappa)
    n_r = math.floor(m_r / (10 + Fraction(100, 2)))
    c_l = math.floor(n_l * Fraction(30, 10))                 # C = N p / d
    c_r = math.floor(n_r * Fraction(10, 100))
    assert (n_l, n_r, c_l, c_r) == (3, 14, 9, 1)
    info, d = o.next_batch()
    assert abs(info["m_l"] - float(m_l)) < 1e-9 and abs(info["m_r"] - float(m_r)) < 1e-9
    assert (info["n_l"], info["n_r"], info["c_l"], info["c_r"]) == (3, 14, 9, 1)
    # The scanners alternate, left first, and each stops at its first refusal:
    #   left  r1: 30 prompt tokens against C_L = 9 -> a chunk of 9;   right r5 decodes (N_R 14 -> 13)
    #   left  r0: C_L is spent -> the left scanner stops;              right r4, then r3 decode
    #   right r2: 20 prompt tokens against C_R = 1 -> a chunk of 1;   right r0: C_R is spent -> stop
    assert (info["n_prefill"], info["n_decode"]) == (2, 3)
    assert list(d["seq_request"]) == [1, 2, 3, 4, 5]          # prefill in admission order, decode in leaf order
    assert list(np.diff(d["row_start"])) == [9, 1, 1, 1, 1]
    assert list(d["kv_len"]) == [9, 1, 34, 36, 41]
    # the same descriptor, every array written out: G's 20 shared tokens hold one whole page, which is
    # numbered first and heads the tables of r3 and r4; then the prefill segments' pages, then the
    # decode sequences' private pages in leaf order
    assert list(d["page_start"]) == [0, 1, 2, 5, 8, 11]
    assert list(d["page_ids"]) == [1, 2, 0, 3, 4, 0, 5, 6, 7, 8, 9]
    assert d["n_nodes"] == 1 and list(d["node_parent"]) == [-1]
    assert list(d["node_page_start"]) == [0, 1] and list(d["node_page_ids"]) == [0]
    assert list(d["node_seq_first"]) == [2] and list(d["node_seq_count"]) == [2]
    assert list(d["seq_leaf_node"]) == [-1, -1, 0, 0, -1]
    assert d["n_pages"] == 10


def test_next_batch_caps_split_the_budgets_in_proportion():
    # the same pool with a prefill cap of 5 tokens and a decode cap of 2 sequences: C_L : C_R = 9 : 1
    # gives 4 and 1, N_L : N_R = 3 : 14 gives 0 and 2, so the right scanner admits r5 and r4 and then
    # stops at r3, before it ever reaches r2
    o = B.BuilderOracle(unit_cost_model(1000), hand_pool())
    info, d = o.next_batch(prefill_budget=5, decode_budget=2)
    assert list(d["seq_request"]) == [1, 4, 5]
    assert list(np.diff(d["row_start"])) == [4, 1, 1]
    assert d["n_nodes"] == 0                                  # one member of G alone shares nothing


def test_emit_numbers_nested_prefix_nodes_by_hand():
    # Three decoding requests share 32 tokens (two pages), two of them 16 more (a third page); a fourth
    # shares nothing.  Trie: root -> P[0,32) -> {Q[32,48) -> {a, b}, c}, d.
    P, Q = list(range(100, 132)), list(range(200, 216))
    reqs = [B.Request(P + Q + [1, 2], d_est=50, n_cached=50 + 7),         # a: kv 58 -> 4 pages
            B.Request(P + Q + [3], d_est=60, n_cached=49 + 30),           # b: kv 80 -> 5 pages
            B.Request(P + [4, 5, 6], d_est=70, n_cached=35),              # c: kv 36 -> 3 pages
            B.Request([9] * 5, d_est=4000, n_cached=20)]                  # d: kv 21 -> 2 pages
    o = B.BuilderOracle(unit_cost_model(10 ** 6), reqs)
    order = o.leaf_order
    assert sorted(order) == [0, 1, 2, 3]
    d = o.emit([], [(r, reqs[r].n_cached) for r in range(4)])
    pos = {r: k for k, r in enumerate(order)}
    assert list(d["seq_request"]) == order
    # node 0 = P: pages 0, 1, members a, b, c; node 1 = Q below it: page 2, members a, b
    assert d["n_nodes"] == 2 and list(d["node_parent"]) == [-1, 0]
    assert list(d["node_page_start"]) == [0, 2, 3] and list(d["node_page_ids"]) == [0, 1, 2]
    assert list(d["node_seq_count"]) == [3, 2]
    assert d["node_seq_first"][0] == min(pos[0], pos[1], pos[2]) and d["node_seq_first"][1] == min(pos[0], pos[1])
    # private pages follow in sequence order, from page 3 on
    n_private = {0: 4 - 3, 1: 5 - 3, 2: 3 - 2, 3: 2}
    nxt = 3
    for k, r in enumerate(order):
        tab = list(d["page_ids"][d["page_start"][k]:d["page_start"][k + 1]])
        shared = [0, 1, 2] if r in (0, 1) else ([0, 1] if r == 2 else [])
        assert tab == shared + list(range(nxt, nxt + n_private[r])), (r, tab)
        nxt += n_private[r]
        assert d["seq_leaf_node"][k] == (1 if r in (0, 1) else (0 if r == 2 else -1))
    assert d["n_pages"] == nxt == 9
    # a prefill chunk of request c's sibling position: segments come first and push the members' indices
    d2 = o.emit([(3, 0, 5)], [(0, reqs[0].n_cached), (1, reqs[1].n_cached)])
    assert d2["n_prefill"] == 1 and list(d2["kv_len"])[0] == 5 and list(d2["row_start"]) == [0, 5, 6, 7]
    # with two members left, P and Q share the same member set: P keeps its two pages, Q adds the third
    assert d2["n_nodes"] == 2 and list(d2["node_seq_first"]) == [1, 1] and list(d2["node_seq_count"]) == [2, 2]
    assert list(d2["node_page_ids"]) == [0, 1, 2] and list(d2["page_ids"][:1]) == [3]


def leaves_in_no_longest_non_increasing_subsequence(vals):
    n = len(vals)
    best, sets = 0, []
    for mask in range(1 << n):
        pick = [i for i in range(n) if mask >> i & 1]
        if all(vals[pick[k]] >= vals[pick[k + 1]] for k in range(len(pick) - 1)):
            if len(pick) > best:
                best, sets = len(pick), [set(pick)]
            elif len(pick) == best:
                sets.append(set(pick))
    in_any = set().union(*sets) if sets else set()
    return [i for i in range(n) if i not in in_any]


@pytest.mark.parametrize("seed", range(150))
def test_split_stops_on_c1_or_c2_brute_force(seed):
    # Section 5.4: the search ends when the leaf densities are non-increasing (C1) or when every
    # remaining split costs more than t (C2), and no leaf is split twice.  Pools of at most six
    # leaves; "remaining split" is taken in the narrowest sense that any reading shares: a leaf
    # that belongs to NO longest non-increasing subsequence of the leaf densities (found by
    # enumeration here) is out of place whichever subsequence one keeps.
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(3, 7))
    pref = [[int(t) for t in rng.integers(0, 50, int(rng.integers(4, 40)))] for _ in range(2)]
    reqs = []
    for _ in range(n):
        g = int(rng.integers(0, 3))
        own = [int(t) for t in rng.integers(50, 1000, int(rng.integers(1, 12)))]
        reqs.append(B.Request((pref[g] if g < 2 else []) + own, d_est=int(rng.choice([2, 5, 50, 400, 3000]))))
    base = B.BuilderOracle(cm(), reqs)
    for t in (10, 25, 10 ** 9):
        o = B.BuilderOracle(cm(), reqs)
        info = o.split(t)
        assert info["n_split"] == len(o.detached) <= n and info["rounds"] <= n
        for r in o.detached:                      # only leaves that shared at most t tokens moved
            assert [x for x in base.nodes if x.req == r][0].start <= t
        dens = [Fraction(10 ** 30) if b == 0 else Fraction(a, b) for a, b in o.leaf_keys()]
        assert info["monotone"] == non_increasing(leaf_density(o))
        if info["monotone"]:
            continue                              # C1
        leaf_of = {nd.req: nd for nd in o.nodes if nd.req >= 0}
        for i in leaves_in_no_longest_non_increasing_subsequence(dens):     # C2
            r = o.leaf_order[i]
            lf = leaf_of[r]
            assert lf.parent == 0 or lf.start > t, "request %d is out of place and could still be split for %d <= %d" % (r, lf.start, t)
