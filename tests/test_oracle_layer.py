"""Pins for the layer oracle: every check here is against something other than
the oracle itself (brute force in pure Python, closed forms, invariants)."""
import math

import numpy as np
import pytest

from oracle import layer as O
from paper_2411_16102_amd import workloads as W


SMALL = W.LayerShape(d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=24)


def small_case(seed=0, **kw):
    b = W.batch_random(seed, **kw)
    t = W.make_tensors(SMALL, b, seed, gains="random")
    return b, t


# ---------------------------------------------------------------------------
# brute force: the whole layer in pure Python loops, dense masked attention
# ---------------------------------------------------------------------------
def brute_layer(shape, t, b):
    d, hq, hkv, dh, F = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn
    T = b.n_rows
    ps = b.page_size
    kp = W.bf16_bits_to_f32(t.k_pool).astype(float)
    vp = W.bf16_bits_to_f32(t.v_pool).astype(float)
    x = t.x.astype(float)
    # per-row sequence and position
    seq_of, pos_of = [], []
    for s in range(b.n_seq):
        n = int(b.row_start[s + 1] - b.row_start[s])
        for j in range(n):
            seq_of.append(s)
            pos_of.append(int(b.kv_len[s]) - n + j)

    def norm(v, g):
        ms = sum(float(a) * float(a) for a in v) / len(v)
        return [float(a) / math.sqrt(ms + shape.rms_eps) * float(gg) for a, gg in zip(v, g)]

    def matvec(v, w):  # v[K] times w[K, N]
        K, N = w.shape
        return [sum(v[k] * float(w[k, n]) for k in range(K)) for n in range(N)]

    def rot(vec, pos):
        out = list(vec)
        half = dh // 2
        for i in range(half):
            ang = pos * shape.rope_theta ** (-2.0 * i / dh)
            c, s = math.cos(ang), math.sin(ang)
            out[i] = vec[i] * c - vec[i + half] * s
            out[i + half] = vec[i + half] * c + vec[i] * s
        return out

    qs, ks, vs = [], [], []
    for r in range(T):
        qkv = matvec(norm(x[r], t.g_attn), t.w_qkv.astype(float))
        qs.append([rot(qkv[h * dh:(h + 1) * dh], pos_of[r]) for h in range(hq)])
        ks.append([rot(qkv[(hq + h) * dh:(hq + h + 1) * dh], pos_of[r]) for h in range(hkv)])
        vs.append([qkv[(hq + hkv + h) * dh:(hq + hkv + h + 1) * dh] for h in range(hkv)])

    # the flattened token stream of the whole batch: every sequence's cached tokens
    # (read through its page table) followed by its new rows; one dense score matrix
    # per head with a block mask
    tok_seq, tok_pos, tok_k, tok_v = [], [], [], []
    for s in range(b.n_seq):
        n = int(b.row_start[s + 1] - b.row_start[s])
        c = int(b.kv_len[s]) - n
        for p in range(c):
            pg = int(b.page_ids[int(b.page_start[s]) + p // ps])
            tok_seq.append(s); tok_pos.append(p)
            tok_k.append(kp[pg, p % ps]); tok_v.append(vp[pg, p % ps])
        for j in range(n):
            r = int(b.row_start[s]) + j
            tok_seq.append(s); tok_pos.append(c + j)
            tok_k.append(np.array(ks[r])); tok_v.append(np.array(vs[r]))
    ntok = len(tok_seq)
    y = np.zeros((T, d))
    grp = hq // hkv
    for r in range(T):
        o = []
        for h in range(hq):
            kh = h // grp
            sc = []
            for j in range(ntok):
                if tok_seq[j] == seq_of[r] and tok_pos[j] <= pos_of[r]:
                    sc.append(sum(qs[r][h][e] * float(tok_k[j][kh][e]) for e in range(dh)) / math.sqrt(dh))
                else:
                    sc.append(None)
            m = max(v for v in sc if v is not None)
            w = [0.0 if v is None else math.exp(v - m) for v in sc]
            z = sum(w)
            o.extend(sum(w[j] * float(tok_v[j][kh][e]) for j in range(ntok)) / z for e in range(dh))
        x1 = [float(x[r][i]) + a for i, a in enumerate(matvec(o, t.w_o.astype(float)))]
        h2 = norm(x1, t.g_ffn)
        gate = matvec(h2, t.w_gate.astype(float))
        up = matvec(h2, t.w_up.astype(float))
        act = [g / (1.0 + math.exp(-g)) * u for g, u in zip(gate, up)]
        y[r] = [a + c2 for a, c2 in zip(x1, matvec(act, t.w_down.astype(float)))]
    return y


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_layer_matches_brute_force(seed):
    b, t = small_case(seed, n_prefill=2, n_decode=4, max_q=6, max_ctx=20, n_roots=1)
    assert b.n_rows <= 64
    got = O.layer_step(SMALL, t, b)["y"]
    ref = brute_layer(SMALL, t, b)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-11)


# ---------------------------------------------------------------------------
# closed forms for the small operators
# ---------------------------------------------------------------------------
def test_rmsnorm_constant_vector():
    g = np.array([0.5, -2.0, 3.0, 1.0])
    for c in (3.0, -0.25):
        out = O.rmsnorm(np.full((1, 4), c), g, 1e-5)
        np.testing.assert_allclose(out[0], g * np.sign(c) / math.sqrt(1 + 1e-5 / c ** 2), rtol=1e-13)
    # 3-4-0-0: mean square 25/4, so the normalised vector is (6/5, 8/5, 0, 0) up to eps
    out = O.rmsnorm(np.array([[3.0, 4.0, 0.0, 0.0]]), np.ones(4), 0.0)
    np.testing.assert_allclose(out[0], [1.2, 1.6, 0.0, 0.0], rtol=1e-14)


def test_rope_closed_forms():
    # dh = 2: a single pair rotated by pos radians (theta^0 = 1), counter-clockwise
    v = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    out = O.rope(v, np.array([0.5, 0.5]), 10000.0)
    np.testing.assert_allclose(out[0, 0], [math.cos(0.5), math.sin(0.5)], rtol=1e-14)
    np.testing.assert_allclose(out[1, 0], [-math.sin(0.5), math.cos(0.5)], rtol=1e-14)
    # dh = 4, theta = 10000: pair (0,2) turns by pos, pair (1,3) by pos / 100
    v = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    out = O.rope(v, np.array([3.0]), 10000.0)[0, 0]
    np.testing.assert_allclose(out, [math.cos(3.0), math.cos(0.03), math.sin(3.0), math.sin(0.03)], rtol=1e-13)
    # position 0 is the identity; pair norms are preserved
    rng = np.random.default_rng(0)
    v = rng.standard_normal((5, 3, 8))
    np.testing.assert_array_equal(O.rope(v, np.zeros(5), 5e5), v)
    r = O.rope(v, np.arange(5) * 7.0, 5e5)
    np.testing.assert_allclose(r[..., :4] ** 2 + r[..., 4:] ** 2, v[..., :4] ** 2 + v[..., 4:] ** 2, rtol=1e-12)


def test_rope_inner_product_depends_on_offset_only():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, 1, 16))
    k = rng.standard_normal((1, 1, 16))
    base = None
    for m, n in [(5, 2), (103, 100), (4003, 4000)]:
        ip = float(np.sum(O.rope(q, np.array([m]), 5e5) * O.rope(k, np.array([n]), 5e5)))
        base = ip if base is None else base
        assert abs(ip - base) < 1e-9


def test_silu_values():
    assert O.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.silu(np.array([1.0, -1.0])), [1 / (1 + math.exp(-1)), -1 / (1 + math.e)], rtol=1e-15)
    assert abs(O.silu(np.array([40.0]))[0] - 40.0) < 1e-12


def test_zero_output_projections_pass_x_through():
    b, t = small_case(3)
    t.w_o[:] = 0
    t.w_down[:] = 0
    np.testing.assert_array_equal(O.layer_step(SMALL, t, b)["y"], t.x.astype(np.float64))


def test_ffn_by_hand():
    # d = F = 2, identity matrices, attention switched off by W_o = 0:
    # y = x + silu(h) * h with h = x / rms(x)
    shape = W.LayerShape(2, 1, 1, 2, 2)
    b = W.assemble_batch(16, [(1, 1, -1)], 0, [], None)
    t = W.make_tensors(shape, b, 0)
    t.w_o[:] = 0
    t.w_gate[:] = np.eye(2); t.w_up[:] = np.eye(2); t.w_down[:] = np.eye(2)
    t.x[:] = [[3.0, -4.0]]
    rms = math.sqrt(12.5 + shape.rms_eps)
    h = [3.0 / rms, -4.0 / rms]
    want = [3.0 + h[0] ** 2 / (1 + math.exp(-h[0])), -4.0 + h[1] ** 2 / (1 + math.exp(-h[1]))]
    np.testing.assert_allclose(O.layer_step(shape, t, b)["y"][0], want, rtol=1e-14)


def test_weight_layout_by_hand():
    # W_qkv columns are [q heads | k heads | v heads], each head dh wide.  One decode
    # row with an empty cache attends only to itself, so o = v for every head; with
    # W_o = identity and the FFN off, y = x + v_head(h // G) stacked over the Q heads.
    shape = W.LayerShape(8, 4, 2, 2, 4)
    b = W.assemble_batch(16, [(1, 1, -1)], 0, [], None)
    t = W.make_tensors(shape, b, 5)
    t.w_down[:] = 0
    t.w_o[:] = np.eye(8)
    res = O.layer_step(shape, t, b)
    xr = t.x[0].astype(float)
    h = xr / math.sqrt(float(np.mean(xr * xr)) + shape.rms_eps)
    v = [sum(h[k] * float(t.w_qkv[k, (4 + 2) * 2 + c]) for k in range(8)) for c in range(4)]  # v: 2 heads x 2
    want = xr + np.array([v[0], v[1], v[0], v[1], v[2], v[3], v[2], v[3]])
    np.testing.assert_allclose(res["y"][0], want, rtol=1e-12)


# ---------------------------------------------------------------------------
# attention special cases
# ---------------------------------------------------------------------------
def test_attention_special_cases():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 4, 8))
    K = rng.standard_normal((9, 2, 8))
    V = rng.standard_normal((9, 2, 8))
    # a single visible key: output is its value, exactly
    o = O.attention(q, K[:1], V[:1], 0)
    for h in range(4):
        np.testing.assert_array_equal(o[0, h], V[0, h // 2])
    # all keys equal: uniform weights, output is the mean value
    Ke = np.repeat(K[:1], 9, axis=0)
    o = O.attention(q, Ke, V, 8)
    for h in range(4):
        np.testing.assert_allclose(o[0, h], V[:, h // 2].mean(axis=0), rtol=1e-12)
    # one dominant logit: output tends to that value row
    Kd = K.copy()
    Kd[5, 0] = 200.0 * q[0, 0] / np.linalg.norm(q[0, 0])
    o = O.attention(q, Kd, V, 8)
    np.testing.assert_allclose(o[0, 0], V[5, 0], atol=1e-9)
    # causality: row j of a 3-row chunk after 6 cached tokens ignores later rows
    q3 = rng.standard_normal((3, 4, 8))
    full = O.attention(q3, K, V, 6)
    for j in range(3):
        alone = O.attention(q3[j:j + 1], K[:7 + j], V[:7 + j], 6 + j)
        np.testing.assert_allclose(full[j], alone[0], rtol=1e-12)


def test_page_resolution_by_planted_keys():
    # Plant, for each decode sequence, one cached token whose key is a huge multiple of
    # that sequence's query direction.  Attention must then return the value stored in
    # the slot (page_ids[page_start + t // 16], t % 16), and V there encodes (seq, t).
    shape = W.LayerShape(16, 2, 1, 8, 8)
    b = W.batch_random(7, n_prefill=0, n_decode=6, max_ctx=80)
    t = W.make_tensors(shape, b, 7)
    res0 = O.layer_step(shape, t, b)
    kp = W.bf16_bits_to_f32(t.k_pool).copy()
    vp = W.bf16_bits_to_f32(t.v_pool).copy()
    rng = np.random.default_rng(7)
    planted = {}
    for s in range(b.n_seq):
        c = int(b.kv_len[s]) - 1
        if c == 0:
            continue
        # private (unshared) cached tokens only, so one plant serves one sequence
        shared = 0
        nd = int(b.seq_leaf_node[s])
        while nd >= 0:
            shared += int(b.node_page_start[nd + 1] - b.node_page_start[nd]) * 16
            nd = int(b.node_parent[nd])
        if shared >= c:
            continue
        tok = int(rng.integers(shared, c))
        pg = int(b.page_ids[int(b.page_start[s]) + tok // 16])
        q = res0["q"][int(b.row_start[s])]  # [Hq, dh] at position c
        # cached keys are stored after RoPE, so a key parallel to the rotated query wins
        kp[pg, tok % 16, 0] = (4.0e3 * q[0] / np.linalg.norm(q[0])).astype(np.float32)
        vp[pg, tok % 16, 0] = np.float32(s * 1000 + tok)
        planted[s] = tok
    assert len(planted) >= 3
    t.k_pool = W.f32_to_bf16_bits(kp)
    t.v_pool = W.f32_to_bf16_bits(vp)
    res = O.layer_step(shape, t, b)
    for s, tok in planted.items():
        o = res["attn"][int(b.row_start[s])][:8]
        want = float(W.round_to_bf16(np.array([s * 1000 + tok], dtype=np.float32))[0])
        np.testing.assert_allclose(o, want, rtol=1e-9)


def test_gqa_head_mapping():
    # values constant per KV head: every query head must return its own group's constant
    shape = W.LayerShape(16, 4, 2, 4, 8)
    b = W.batch_decode_only(2, 20, seed=1)
    t = W.make_tensors(shape, b, 1)
    vp = np.zeros(t.v_pool.shape, dtype=np.float32)
    vp[:, :, 0, :] = 1.0
    vp[:, :, 1, :] = -2.0
    t.v_pool = W.f32_to_bf16_bits(vp)
    t.w_qkv[:, (4 + 2) * 4:] = 0.0          # this step's v is zero
    res = O.layer_step(shape, t, b)
    # the new token's v is 0, so each head returns const * (1 - weight of the new token)
    a = res["attn"].reshape(-1, 4, 4)
    assert np.all(a[:, 0] > 0) and np.all(a[:, 1] > 0) and np.all(a[:, 2] < 0) and np.all(a[:, 3] < 0)
    np.testing.assert_allclose(a[:, 2] / a[:, 2, :1], 1.0, rtol=1e-12)


# ---------------------------------------------------------------------------
# invariants
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed", [0, 4])
def test_shared_and_expanded_kv_agree_bitwise(seed):
    b, t = small_case(seed)
    e, src = W.expand_batch(b)
    te = W.make_tensors(SMALL, b, seed, gains="random")
    te.k_pool = t.k_pool[np.maximum(src, 0)]
    te.v_pool = t.v_pool[np.maximum(src, 0)]
    a = O.layer_step(SMALL, t, b)
    c = O.layer_step(SMALL, te, e)
    np.testing.assert_array_equal(a["y"], c["y"])
    np.testing.assert_array_equal(a["attn"], c["attn"])


def test_request_order_only_permutes_rows():
    b, t = small_case(5, n_prefill=3, n_decode=5, n_roots=0)
    res = O.layer_step(SMALL, t, b)
    # reverse the prefill segments among themselves and the decode sequences among themselves
    order = list(range(b.n_prefill))[::-1] + list(range(b.n_prefill, b.n_seq))[::-1]
    q_len = b.q_len()
    seqs = [(int(q_len[s]), int(b.kv_len[s]), -1) for s in order]
    b2 = W.assemble_batch(16, seqs, b.n_prefill, [], None)
    # same physical contents: copy each sequence's pages to its new private pages
    t2 = W.make_tensors(SMALL, b, 5, gains="random")
    kp = np.zeros((b2.n_pages,) + t.k_pool.shape[1:], dtype=np.uint16)
    vp = np.zeros_like(kp)
    rows = []
    for new_s, s in enumerate(order):
        n = int(b.page_start[s + 1] - b.page_start[s])
        old = b.page_ids[int(b.page_start[s]):int(b.page_start[s]) + n]
        new = b2.page_ids[int(b2.page_start[new_s]):int(b2.page_start[new_s]) + n]
        kp[new] = t.k_pool[old]
        vp[new] = t.v_pool[old]
        rows.extend(range(int(b.row_start[s]), int(b.row_start[s + 1])))
    t2.k_pool, t2.v_pool = kp, vp
    t2.x = t.x[rows]
    res2 = O.layer_step(SMALL, t2, b2)
    np.testing.assert_allclose(res2["y"], res["y"][rows], rtol=1e-12, atol=1e-13)


def test_chunked_prefill_equals_one_shot():
    # a 48-row prefill in one step == 20 rows, then 28 rows over the cached first chunk
    rng = np.random.default_rng(11)
    whole = W.assemble_batch(16, [(48, 48, -1)], 1, [], None)
    t = W.make_tensors(SMALL, whole, 11, gains="random")
    full = O.layer_step(SMALL, t, whole)
    first = W.assemble_batch(16, [(20, 20, -1)], 1, [], None)
    first.n_pages = whole.n_pages
    t1 = W.make_tensors(SMALL, whole, 11, gains="random")
    t1.x = t.x[:20]
    r1 = O.layer_step(SMALL, t1, first)
    kp, vp = O.append_kv(first, r1, t.k_pool, t.v_pool)
    second = W.assemble_batch(16, [(28, 48, -1)], 1, [], None)
    t2 = W.make_tensors(SMALL, whole, 11, gains="random")
    t2.x = t.x[20:]
    t2.k_pool, t2.v_pool = kp, vp
    r2 = O.layer_step(SMALL, t2, second)
    np.testing.assert_allclose(r1["y"], full["y"][:20], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r2["y"], full["y"][20:], rtol=1e-12, atol=1e-13)
    # the appended pool equals what the one-shot step appends
    kpf, vpf = O.append_kv(whole, full, t.k_pool, t.v_pool)
    kp2, vp2 = O.append_kv(second, r2, kp, vp)
    np.testing.assert_allclose(kp2[:3], kpf[:3], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(vp2[:3], vpf[:3], rtol=1e-12, atol=1e-13)


def test_one_row_prefill_chunk_equals_decode():
    b = W.assemble_batch(16, [(1, 37, -1)], 1, [], None)   # as a prefill segment
    b2 = W.assemble_batch(16, [(1, 37, -1)], 0, [], None)  # as a decode sequence
    t = W.make_tensors(SMALL, b, 2)
    np.testing.assert_array_equal(O.layer_step(SMALL, t, b)["y"], O.layer_step(SMALL, t, b2)["y"])


def test_row_subset_matches_full():
    b, t = small_case(6)
    full = O.layer_step(SMALL, t, b)["y"]
    rows = [0, b.n_rows // 2, b.n_rows - 1]
    sub = O.layer_step(SMALL, t, b, rows=rows)["y"]
    np.testing.assert_allclose(sub[rows], full[rows], rtol=1e-12, atol=1e-13)
    assert np.isnan(sub[[r for r in range(b.n_rows) if r not in rows]]).all()


def test_lse_merge_is_associative():
    # splitting the keys of one query into any groups and merging partial softmax states
    # (m, l, acc) reproduces the one-pass result: the identity the GPU's prefix-aware
    # kernel relies on, checked here against the oracle's plain attention
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 1, 8))
    K = rng.standard_normal((40, 1, 8)) * 3
    V = rng.standard_normal((40, 1, 8))
    ref = O.attention(q, K, V, 39)[0, 0]
    for cuts in ([0, 40], [0, 7, 40], [0, 16, 17, 33, 40]):
        m, l, acc = -math.inf, 0.0, np.zeros(8)
        for a, c in zip(cuts[:-1], cuts[1:]):
            s = (K[a:c, 0] @ q[0, 0]) / math.sqrt(8)
            mp = float(s.max()); p = np.exp(s - mp)
            lp, ap = float(p.sum()), p @ V[a:c, 0]
            mn = max(m, mp)
            l = l * math.exp(m - mn) + lp * math.exp(mp - mn)
            acc = acc * math.exp(m - mn) + ap * math.exp(mp - mn)
            m = mn
        np.testing.assert_allclose(acc / l, ref, rtol=1e-12)


def test_bf16_storage_mode_is_close_and_representable():
    b, t = small_case(8)
    a = O.layer_step(SMALL, t, b)["y"]
    r = O.layer_step(SMALL, t, b, storage="bf16")["y"]
    np.testing.assert_array_equal(W.round_to_bf16(r.astype(np.float32)).astype(np.float64), r)
    assert np.max(np.abs(a - r)) / np.max(np.abs(a)) < 2e-2
