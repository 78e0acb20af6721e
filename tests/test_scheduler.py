"""The multi-step driver: its oracle against brute-force properties, and the C++ scheduler against
the oracle, descriptor by descriptor, bit for bit, over whole pools served to completion.  No GPU."""
import numpy as np
import pytest

from oracle import builder as OB
from oracle import scheduler as OS
from paper_2411_16102_amd import binding, workloads as W

HW = dict(p_model=8_030_000_000, kv_bytes=1024 * 32 * 4, compute=2.5e15, bandwidth=8.0e12)


def pool(seed, n_groups=4, per_group=5, n_fresh=8, two_level=True, dup=True):
    """Prompts with shared system prefixes (some nested, some ending on a page boundary), a prompt
    that is the prefix of another and an exact duplicate; estimates off by up to 3x either way."""
    rng = np.random.default_rng(seed)
    toks, d_true = [], []
    for g in range(n_groups):
        prefix = [int(t) for t in rng.integers(10, 5000, int(rng.choice([16, 32, 40, 57, 64, 100])))]
        mid = [int(t) for t in rng.integers(10, 5000, int(rng.choice([8, 16, 24])))] if two_level and g % 2 else []
        for k in range(per_group):
            own = [int(t) for t in rng.integers(10, 5000, int(rng.integers(1, 40)))]
            toks.append(prefix + (mid if k % 2 else []) + own)
            d_true.append(int(rng.choice([1, 2, 3, 8, 30, 90])))
    for _ in range(n_fresh):
        toks.append([int(t) for t in rng.integers(10, 5000, int(rng.integers(5, 150)))])
        d_true.append(int(rng.choice([1, 2, 5, 12])))
    if dup:
        toks.append(list(toks[0]))            # exact duplicate
        d_true.append(4)
        toks.append(list(toks[1][:32]))       # a prompt that is a prefix of another, ending on a page boundary
        d_true.append(6)
    d_est = [max(1, int(round(d * float(np.exp(0.6 * rng.standard_normal()))))) for d in d_true]
    return toks, d_est, d_true


def make_both(toks, d_est, d_true, mem_tokens, budget, n_pages, order=None, split_t=0, **kw):
    cm = OB.CostModel(mem_bytes=mem_tokens * HW["kv_bytes"], page_size=16, **HW)
    ot = OB.BuilderOracle(cm, [OB.Request(t, d, 0) for t, d in zip(toks, d_est)])
    b = binding.Builder(HW["p_model"], HW["kv_bytes"], HW["compute"], HW["bandwidth"], mem_tokens * HW["kv_bytes"], 16)
    for t, d in zip(toks, d_est):
        b.add(t, d, 0)
    b.finalize()
    if split_t:
        ot.split(split_t)
        b.split(split_t)
    o = OS.SchedulerOracle(ot, d_true, mem_tokens, budget, n_pages, order=order, **kw)
    s = binding.Scheduler(b, d_true, mem_tokens, budget, n_pages, order=order, **kw)
    return o, s


def same(a, b):
    assert set(a) == set(b)
    for k in a:
        if isinstance(a[k], np.ndarray):
            assert np.array_equal(a[k], b[k]), (k, a[k], b[k])
        else:
            assert a[k] == b[k], k


def check_descriptor(d, toks, state, host_layer):
    """What must hold for every step, whatever the admission policy: the library's validator accepts
    the descriptor; every page of every table holds the tokens that table says (tracked in `state`:
    page -> the (request-independent) token sequence written into it so far)."""
    batch = W.Batch(page_size=16, **{k: v for k, v in d.items() if k != "seq_request"})
    assert host_layer.validate(batch) == 0, host_layer.last_error()
    q = np.diff(d["row_start"])
    for s_ in range(d["n_seq"]):
        r = int(d["seq_request"][s_])
        kv, n = int(d["kv_len"][s_]), int(q[s_])
        tab = d["page_ids"][d["page_start"][s_]:d["page_start"][s_ + 1]]
        p = len(toks[r])
        for pos in range(kv):
            pg, sl = int(tab[pos // 16]), pos % 16
            tok = toks[r][pos] if pos < p else ("out", r, pos)      # prompt token, or this request's own output
            if pos >= kv - n:
                state[(pg, sl)] = tok                                 # written this step
            else:
                assert state.get((pg, sl)) == tok, "request %d reads position %d from a page that holds something else" % (r, pos)


@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("mode", ["blend", "blend_split", "given_order", "row_multiple"])
def test_cpp_scheduler_matches_the_oracle_step_by_step(seed, mode):
    toks, d_est, d_true = pool(seed)
    kw = {}
    order = None
    if mode == "given_order":
        order = [int(i) for i in np.random.default_rng(seed).permutation(len(toks))]
    if mode == "row_multiple":
        kw = dict(row_multiple=8, relocate_pct=0)
    o, s = make_both(toks, d_est, d_true, mem_tokens=700, budget=96, n_pages=120, order=order,
                     split_t=40 if mode == "blend_split" else 0, **kw)
    host_layer = binding.Layer(W.TINY, device=-1)
    state = {}
    steps = 0
    while True:
        want, got = o.next_step(), s.next_step()
        if want is None:
            assert got is None
            break
        same(want, got)
        check_descriptor(got, toks, state, host_layer)
        steps += 1
        assert steps < 5000
    st = s.stats()
    for k, v in o.stats.items():
        assert st[k] == v, k
    assert st["finished"] == len(toks) and st["tokens_out"] == sum(d_true)
    assert st["peak_pages"] <= 120 and len(o.free) == 120          # every page came back
    assert st["mem_left"] + st["mem_right"] == 700


def test_scheduler_hand_worked_steps():
    # Three requests, unit-size numbers.  a and b share a 32-token prefix (two pages); c is alone.
    # Budget 40 rows, memory for everything.  One scanner (given order a, b, c).
    P = list(range(100, 132))
    toks = [P + [1, 2, 3], P + [4], [7] * 20]
    o, s = make_both(toks, [2, 2, 2], [2, 3, 1], mem_tokens=1000, budget=40, n_pages=16, order=[0, 1, 2])
    # step 1: a is admitted and owns the shared segment; 35 rows.  b needs a segment that a is still
    # computing: it waits, and the scanner stops (c is behind b in the order).
    d = s.next_step(); same(o.next_step(), d)
    assert list(d["seq_request"]) == [0] and list(d["kv_len"]) == [35] and list(d["page_ids"]) == [0, 1, 2]
    # step 2: a decodes at position 35 (its second token; the first came with the last prompt row);
    # b starts behind the two shared pages: 1 row at position 32; c: 20 rows.  Pages: b's private
    # page is 3, c's are 4 and 5.
    d = s.next_step(); same(o.next_step(), d)
    assert list(d["seq_request"]) == [1, 2, 0]
    assert list(d["kv_len"]) == [33, 20, 36] and list(np.diff(d["row_start"])) == [1, 20, 1]
    assert list(d["page_ids"]) == [0, 1, 3, 4, 5, 0, 1, 2]
    assert d["n_nodes"] == 0                        # one decode member only
    # a has produced its 2 tokens and c its 1: both leave; their private pages 2, 4, 5 are free again.
    # step 3: b decodes at position 33, alone.
    d = s.next_step(); same(o.next_step(), d)
    assert list(d["seq_request"]) == [1] and list(d["kv_len"]) == [34] and list(d["page_ids"]) == [0, 1, 3]
    d = s.next_step(); same(o.next_step(), d)
    assert list(d["kv_len"]) == [35]
    assert s.next_step() is None and o.next_step() is None
    assert s.stats()["prompt_tokens_skipped"] == 32 and s.stats()["steps"] == 4


def test_two_decoders_below_a_segment_form_a_prefix_node():
    P = list(range(100, 148))                       # 48 tokens: three pages
    toks = [P + [1], P + [2, 3]]
    o, s = make_both(toks, [5, 5], [5, 5], mem_tokens=1000, budget=64, n_pages=16, order=[0, 1])
    descs = []
    while True:
        d = s.next_step()
        w = o.next_step()
        if d is None:
            break
        same(w, d)
        descs.append(d)
    both = [d for d in descs if d["n_seq"] - d["n_prefill"] == 2]
    assert both, "the two requests never decoded together"
    for d in both:
        assert d["n_nodes"] == 1 and list(d["node_page_ids"]) == [0, 1, 2] and list(d["node_seq_count"]) == [2]
        assert list(d["seq_leaf_node"][d["n_prefill"]:]) == [0, 0]
        for s_ in range(d["n_prefill"], d["n_seq"]):
            assert list(d["page_ids"][d["page_start"][s_]:d["page_start"][s_] + 3]) == [0, 1, 2]


def test_pool_exhaustion_is_an_error_code():
    toks, d_est, d_true = pool(3, dup=False)
    _, s = make_both(toks, d_est, d_true, mem_tokens=5000, budget=256, n_pages=6)
    with pytest.raises(binding.BlendStepError) as ei:
        for _ in range(100):
            if s.next_step() is None:
                break
    assert ei.value.code == -2 and "exhausted" in str(ei.value)
