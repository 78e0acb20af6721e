"""Parity of the HIP path with the CPU oracle, through the C ABI, at sizes the
oracle finishes in seconds (several tiles and ragged tails included).

Tolerances: the one rule of tests/parity_rule.py (max relative error 2e-2 over a tensor; mean
absolute error against the exact oracle rounded to bfloat16 at most 1e-3, or 1.25 times the error
that bfloat16 storage alone causes at that shape where that is larger).  Integer work (page and
slot of every appended row, which pool elements change) is compared exactly.
"""
import numpy as np
import pytest

from oracle import layer as O
from paper_2411_16102_amd import workloads as W
from parity_rule import MAE, MAXREL, check, errs

pytestmark = pytest.mark.gpu


def to_np(t):
    return t.float().cpu().numpy().astype(np.float64)


def run_step(lib, shape, batch, tens, flags=0):
    import torch
    layer = lib.Layer(shape, device=0)
    dev = layer.upload(tens, batch)
    y = layer.blend_step(dev, batch, flags=flags)
    torch.cuda.synchronize()
    k, v = layer.unpack_pool(dev.kv_pool, dev.n_pages)
    return to_np(y), to_np(k), to_np(v), layer


def check_step(lib, shape, batch, tens, flags=0):
    ref = O.layer_step(shape, tens, batch)
    diag = O.layer_step(shape, tens, batch, storage="bf16")
    y, k, v, layer = run_step(lib, shape, batch, tens, flags)
    check(y, ref["y"], diag["y"], "rows=%d" % batch.n_rows)
    # KV append: exactly the destination slots change, and they hold k, v of the rows
    k0 = W.bf16_bits_to_f32(tens.k_pool).astype(np.float64)
    v0 = W.bf16_bits_to_f32(tens.v_pool).astype(np.float64)
    written = np.zeros(k0.shape[:2], dtype=bool)
    written[ref["dest"][:, 0], ref["dest"][:, 1]] = True
    assert np.array_equal(k[~written], k0[~written]), "a slot outside the append destinations changed (K)"
    assert np.array_equal(v[~written], v0[~written]), "a slot outside the append destinations changed (V)"
    kn = k[ref["dest"][:, 0], ref["dest"][:, 1]]
    vn = v[ref["dest"][:, 0], ref["dest"][:, 1]]
    check(kn, ref["k_new"], diag["k_new"], "appended keys")
    check(vn, ref["v_new"], diag["v_new"], "appended values")
    pg, sl = layer.resolve_rows(batch)
    assert np.array_equal(pg, ref["dest"][:, 0]) and np.array_equal(sl, ref["dest"][:, 1])
    return y, ref


# ---------------------------------------------------------------------------
# stand-alone operators
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,k", [(136, 512, 256), (300, 264, 688), (1, 8, 8), (1030, 1544, 520), (2048, 1024, 512),
                                   # at most 256 / 128 rows and a row of tiles that fills the chip: the deep weight ring
                                   (200, 16512, 520), (256, 16384, 192), (100, 33000, 328), (128, 32768, 1024)])
def test_gemm_nt(lib, m, n, k):
    import torch
    rng = np.random.default_rng(m + n + k)
    a = W.round_to_bf16(rng.standard_normal((m, k), dtype=np.float32))
    b = W.round_to_bf16(rng.standard_normal((n, k), dtype=np.float32) * 0.05)
    layer = lib.Layer(W.TINY, device=0)
    ta = torch.from_numpy(a).cuda().to(torch.bfloat16)
    tb = torch.from_numpy(b).cuda().to(torch.bfloat16)
    c = to_np(layer.gemm_nt(ta, tb))
    ref = a.astype(np.float64) @ b.astype(np.float64).T
    maxrel, mae = errs(c, ref)
    # a bf16 result is within half an ulp (2^-9 relative) of the exact value plus fp32 accumulation error
    assert np.max(np.abs(c - ref) / (np.abs(ref) + 1e-3 * np.max(np.abs(ref)))) < 6e-3
    assert maxrel < 4e-3


@pytest.mark.parametrize("m,n,k", [(2600, 4104, 520),    # 187 tiles for 256 workgroups: every tile cut along K
                                   (4096, 4096, 192),    # 256 tiles: one whole round, nothing shared
                                   (4100, 5000, 328),    # 340 tiles: all shared, more than a tile's worth each
                                   (5000, 7000, 200),    # 560 tiles: a round of whole tiles, then 304 shared ones
                                   (300, 704, 8200),     # 6 tiles, 129 k-tiles each: dozens of parts per tile
                                   (256, 256, 64), (1, 8, 8)])
def test_gemm_nt_on_shared_tiles(lib, m, n, k):
    # tile shape 6: persistent workgroups, the tiles of the last rounds cut along K; whoever arrives
    # last at a tile adds its parts up in a fixed order, so two runs agree bit for bit
    import torch
    rng = np.random.default_rng(m + n + k)
    a = W.round_to_bf16(rng.standard_normal((m, k), dtype=np.float32))
    b = W.round_to_bf16(rng.standard_normal((n, k), dtype=np.float32) * 0.05)
    layer = lib.Layer(W.TINY, device=0)
    layer.set_gemm_tiles(6)
    ta = torch.from_numpy(a).cuda().to(torch.bfloat16)
    tb = torch.from_numpy(b).cuda().to(torch.bfloat16)
    c1 = layer.gemm_nt(ta, tb)
    c2 = layer.gemm_nt(ta, tb)       # also: the arrival counters were left at zero
    torch.cuda.synchronize()
    assert torch.equal(c1, c2)
    c = to_np(c1)
    ref = a.astype(np.float64) @ b.astype(np.float64).T
    maxrel, mae = errs(c, ref)
    assert np.max(np.abs(c - ref) / (np.abs(ref) + 1e-3 * np.max(np.abs(ref)))) < 6e-3
    assert maxrel < 4e-3


@pytest.mark.parametrize("shape", [W.LayerShape(1024, 8, 2, 128, 2056), W.LayerShape(512, 8, 2, 64, 33024)])
def test_layer_step_on_shared_tiles(lib, shape):
    # every GEMM of the step, with its fused epilogue, on shared tiles (ragged in every dimension)
    import torch
    batch = W.assemble_batch(16, [(700, 700, -1), (391, 500, -1)] + [(1, 200 + 7 * i, -1) for i in range(50)], 2,
                             [], np.random.default_rng(5))
    tens = W.make_tensors(shape, batch, 5, gains="random")
    ref = O.layer_step(shape, tens, batch)
    diag = O.layer_step(shape, tens, batch, storage="bf16")
    layer = lib.Layer(shape, device=0)
    layer.set_gemm_tiles(6)
    dev = layer.upload(tens, batch)
    y = layer.blend_step(dev, batch)
    torch.cuda.synchronize()
    check(to_np(y), ref["y"], diag["y"], "shared tiles")
    k, v = layer.unpack_pool(dev.kv_pool, dev.n_pages)
    k, v = to_np(k), to_np(v)
    check(k[ref["dest"][:, 0], ref["dest"][:, 1]], ref["k_new"], diag["k_new"], "appended keys")
    check(v[ref["dest"][:, 0], ref["dest"][:, 1]], ref["v_new"], diag["v_new"], "appended values")


def attention_reference(shape, batch, q, k_pool, v_pool, storage="exact"):
    out = np.zeros((batch.n_rows, shape.n_q_heads * shape.head_dim))
    for s in range(batch.n_seq):
        r0, r1 = int(batch.row_start[s]), int(batch.row_start[s + 1])
        L = int(batch.kv_len[s])
        K, V = O.gather_kv(batch, s, L, k_pool, v_pool)
        o = O.attention(q[r0:r1].reshape(r1 - r0, shape.n_q_heads, shape.head_dim), K, V, L - (r1 - r0), storage)
        out[r0:r1] = o.reshape(r1 - r0, -1)
    return out


def check_attention(shape, batch, q, tens, out, what="attention"):
    ref = attention_reference(shape, batch, q.astype(np.float64), tens.k_pool, tens.v_pool)
    diag = attention_reference(shape, batch, q.astype(np.float64), tens.k_pool, tens.v_pool, "bf16")
    diag = W.round_to_bf16(diag.astype(np.float32)).astype(np.float64)   # the output is stored in bfloat16 too
    check(out, ref, diag, what)


@pytest.mark.parametrize("shape", [W.LayerShape(256, 4, 2, 64, 688), W.LayerShape(512, 8, 2, 128, 256),
                                   W.LayerShape(512, 8, 1, 128, 256), W.LayerShape(256, 4, 4, 64, 256)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_attention_alone(lib, shape, seed):
    import torch
    batch = W.batch_random(seed, n_prefill=4, n_decode=40, max_q=100, max_ctx=700, n_roots=3)
    tens = W.make_tensors(shape, batch, seed)
    rng = np.random.default_rng(seed)
    q = W.round_to_bf16(rng.standard_normal((batch.n_rows, shape.n_q_heads * shape.head_dim), dtype=np.float32))
    layer = lib.Layer(shape, device=0)
    layer.set_chunk_pages(4)  # several chunks per node and per tail
    pool = layer.pack_pool(tens.k_pool, tens.v_pool)
    tq = torch.from_numpy(q).cuda().to(torch.bfloat16)
    out = to_np(layer.attention(batch, tq, pool, batch.n_pages))
    check_attention(shape, batch, q, tens, out)


@pytest.mark.parametrize("shape", [W.LayerShape(256, 4, 2, 64, 256), W.LayerShape(512, 8, 2, 128, 256),
                                   W.LayerShape(1024, 8, 1, 128, 256)])
@pytest.mark.parametrize("members", [[2, 9], [5, 17, 33], [8, 16, 70]])
def test_attention_node_member_counts(lib, shape, members):
    # prefix nodes whose members fill one to several blocks of 16 query rows, some of
    # them partly: a root of 35 tokens per member count, one child node under the first
    import torch
    nodes, seqs = [], [(7, 40, -1)]
    rng = np.random.default_rng(sum(members))
    for k, n in enumerate(members):
        root = len(nodes)
        nodes.append((-1, 2 + k))
        leaf = root
        if k == 0:
            nodes.append((root, 3))
            leaf = root + 1
        for j in range(n):
            shared = 16 * ((2 + k) + (3 if leaf != root else 0))
            nd = leaf if j < (n + 1) // 2 or leaf == root else root
            sh = shared if nd == leaf else 16 * (2 + k)
            seqs.append((1, sh + 1 + int(rng.integers(0, 90)), nd))
    # members of the child node come first within the root's run: already so by construction
    batch = W.assemble_batch(16, seqs, 1, nodes, rng)
    tens = W.make_tensors(shape, batch, 5)
    q = W.round_to_bf16(rng.standard_normal((batch.n_rows, shape.n_q_heads * shape.head_dim), dtype=np.float32))
    layer = lib.Layer(shape, device=0)
    pool = layer.pack_pool(tens.k_pool, tens.v_pool)
    out = to_np(layer.attention(batch, torch.from_numpy(q).cuda().to(torch.bfloat16), pool, batch.n_pages))
    check_attention(shape, batch, q, tens, out)


@pytest.mark.parametrize("root_pages,n_members", [(20, 40), (14, 41)])
def test_attention_wide_items_alternate_with_narrow_ones(lib, root_pages, n_members):
    # one long shared root cut into chunks of two pages, short private tails: the workgroups of
    # 64-row items are more than a third of the launch, so the grid takes its mixed order (some
    # wide workgroups ahead, then one wide and two narrow in turn, then what is left)
    import torch
    shape = W.LayerShape(512, 8, 2, 128, 256)
    rng = np.random.default_rng(root_pages * 100 + n_members)
    nodes = [(-1, root_pages)]
    seqs = [(7, 40, -1)] + [(1, 16 * root_pages + 1 + int(rng.integers(0, 30)), 0) for _ in range(n_members)]
    batch = W.assemble_batch(16, seqs, 1, nodes, rng)
    tens = W.make_tensors(shape, batch, 11)
    q = W.round_to_bf16(rng.standard_normal((batch.n_rows, shape.n_q_heads * shape.head_dim), dtype=np.float32))
    layer = lib.Layer(shape, device=0)
    layer.set_chunk_pages(2)
    pool = layer.pack_pool(tens.k_pool, tens.v_pool)
    out = to_np(layer.attention(batch, torch.from_numpy(q).cuda().to(torch.bfloat16), pool, batch.n_pages))
    check_attention(shape, batch, q, tens, out)


def test_attention_ignores_stale_slots(lib):
    # slots past kv_len in the last page hold NaN bit patterns: they must never reach the output
    import torch
    shape = W.LayerShape(256, 4, 2, 64, 688)
    batch = W.assemble_batch(16, [(5, 21, -1), (1, 35, -1), (1, 17, -1)], 1, [], None)
    tens = W.make_tensors(shape, batch, 3)
    kp, vp = tens.k_pool.copy(), tens.v_pool.copy()
    for s in range(batch.n_seq):
        L = int(batch.kv_len[s])
        pg = int(batch.page_ids[int(batch.page_start[s]) + (L - 1) // 16])
        kp[pg, L % 16:] = 0x7FC0 if L % 16 else kp[pg, L % 16:]
        vp[pg, L % 16:] = 0x7FC0 if L % 16 else vp[pg, L % 16:]
    rng = np.random.default_rng(0)
    q = W.round_to_bf16(rng.standard_normal((batch.n_rows, 256), dtype=np.float32))
    layer = lib.Layer(shape, device=0)
    pool = layer.pack_pool(kp, vp)
    out = to_np(layer.attention(batch, torch.from_numpy(q).cuda().to(torch.bfloat16), pool, batch.n_pages))
    assert np.isfinite(out).all()
    ref = attention_reference(shape, batch, q.astype(np.float64), tens.k_pool, tens.v_pool)
    assert errs(out, ref)[0] <= MAXREL


# ---------------------------------------------------------------------------
# the whole step
# ---------------------------------------------------------------------------
def test_tiny_config(lib):
    batch = W.batch_tiny(0)
    tens = W.make_tensors(W.TINY, batch, 0)
    check_step(lib, W.TINY, batch, tens)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
@pytest.mark.parametrize("flags", [0, 1])
def test_random_batches_tiny_shape(lib, seed, flags):
    batch = W.batch_random(seed, n_prefill=3, n_decode=20, max_q=90, max_ctx=400, n_roots=2)
    tens = W.make_tensors(W.TINY, batch, seed, gains="random")
    check_step(lib, W.TINY, batch, tens, flags)


@pytest.mark.parametrize("seed", [0, 1])
def test_random_batches_head_dim_128(lib, seed):
    shape = W.LayerShape(512, 8, 2, 128, 1288)
    batch = W.batch_random(10 + seed, n_prefill=4, n_decode=30, max_q=150, max_ctx=600, n_roots=3)
    tens = W.make_tensors(shape, batch, seed, gains="random")
    check_step(lib, shape, batch, tens)


def test_many_rows_use_large_tiles(lib):
    # enough rows for the 256x256-tile instances, ragged in every dimension
    shape = W.LayerShape(1024, 8, 2, 128, 2056)
    batch = W.assemble_batch(16, [(700, 700, -1), (391, 500, -1)] + [(1, 200 + 7 * i, -1) for i in range(50)], 2,
                             [], np.random.default_rng(5))
    tens = W.make_tensors(shape, batch, 5)
    check_step(lib, shape, batch, tens)


@pytest.mark.parametrize("n_decode,q_rows", [(60, 40), (120, 80), (97, 0)])
def test_few_rows_take_the_deep_weight_ring(lib, n_decode, q_rows):
    # at most 128 / 256 rows: the QKV, output and down projections run as k-ranges of a single
    # row of tiles on the pipeline with its own look-ahead for the weight panel
    shape = W.LayerShape(1024, 8, 2, 128, 2048)
    seqs = ([(q_rows, q_rows + 30, -1)] if q_rows else []) + [(1, 50 + 11 * i, -1) for i in range(n_decode)]
    batch = W.assemble_batch(16, seqs, 1 if q_rows else 0, [], np.random.default_rng(n_decode))
    tens = W.make_tensors(shape, batch, 7, gains="random")
    check_step(lib, shape, batch, tens)


@pytest.mark.parametrize("d_model,d_ffn", [(256, 32768), (512, 33024)])
def test_rounds_of_full_tiles_in_gate_up(lib, d_model, d_ffn):
    # 512 rows and a wide FFN: the gate/up GEMM has two whole rounds of full 256x256 tiles (four and
    # eight k-tiles per tile); the second shape adds a last round that goes out on the small tiles
    shape = W.LayerShape(d_model, 4, 2, 64, d_ffn)
    batch = W.assemble_batch(16, [(300, 300, -1), (150, 180, -1)] + [(1, 20 + 3 * i, -1) for i in range(62)], 2,
                             [], np.random.default_rng(9))
    assert batch.n_rows == 512
    tens = W.make_tensors(shape, batch, 9)
    check_step(lib, shape, batch, tens)


def test_decode_only_and_prefill_only(lib):
    for batch in (W.batch_decode_only(33, 130, seed=2), W.batch_prefill_only(3, 75, seed=2)):
        tens = W.make_tensors(W.TINY, batch, 2)
        check_step(lib, W.TINY, batch, tens)


def test_degenerate_batches(lib):
    import torch
    shape = W.TINY
    layer = lib.Layer(shape, device=0)
    # an empty batch is accepted and touches nothing
    empty = W.assemble_batch(16, [], 0, [], None)
    tens = W.make_tensors(shape, W.batch_tiny(0), 0)
    dev = layer.upload(tens, W.batch_tiny(0))
    y = torch.full_like(dev.x, 7.0)
    layer.blend_step(dev, empty, y=y)
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
    # one decode sequence whose context is its own token: attention returns its value vector
    # (softmax over one score is 1), so this reduces to the dense part of the layer
    one = W.assemble_batch(16, [(1, 1, -1)], 0, [], None)
    check_step(lib, shape, one, W.make_tensors(shape, one, 1))
    # a one-row prefill chunk behind a cached context, contexts that end exactly on a page
    # boundary, and one that starts a fresh page with this step's row
    edge = W.assemble_batch(16, [(1, 48, -1), (16, 32, -1), (3, 35, -1), (1, 16, -1), (1, 17, -1), (1, 33, -1)], 3, [],
                            np.random.default_rng(5))
    check_step(lib, shape, edge, W.make_tensors(shape, edge, 2, gains="random"))


def test_ragged_prefill_segments(lib):
    # segments of 1, 31, 32, 33, 64, 65 and 97 rows (a wavefront of prefill attention owns 64) behind
    # cached contexts that end on and off page and block boundaries
    shape = W.LayerShape(512, 8, 2, 128, 256)
    segs = [(1, 48, -1), (31, 31, -1), (32, 96, -1), (33, 33, -1), (64, 200, -1), (65, 129, -1), (97, 1000, -1)]
    batch = W.assemble_batch(16, segs + [(1, 77, -1)], len(segs), [], np.random.default_rng(11))
    check_step(lib, shape, batch, W.make_tensors(shape, batch, 6, gains="random"))


def test_contexts_up_to_the_last_position(lib):
    # the longest contexts the default RoPE table (16384 positions) admits: a prefill chunk whose
    # last row sits at the last position, decode sequences there and one page short of it, two of
    # them behind a shared prefix of 1000 pages (split over many chunks of the decode kernel)
    shape = W.TINY
    top = 16384
    batch = W.assemble_batch(16, [(70, top, -1), (1, top, -1), (1, top, 0), (1, top - 16, 0), (1, 5000, -1)], 1,
                             [(-1, 1000)], np.random.default_rng(9))
    check_step(lib, shape, batch, W.make_tensors(shape, batch, 4, gains="random"))


@pytest.mark.parametrize("shape", [W.LayerShape(512, 16, 1, 64, 256), W.LayerShape(256, 4, 4, 64, 344)])
def test_group_sizes_sixteen_and_one(lib, shape):
    # 16 query heads per KV head (one member fills a decode work item) and plain multi-head attention
    batch = W.batch_random(8, n_prefill=2, n_decode=14, max_q=40, max_ctx=260, n_roots=2)
    check_step(lib, shape, batch, W.make_tensors(shape, batch, 8))


def test_shared_and_expanded_kv_agree(lib):
    batch = W.batch_random(21, n_prefill=2, n_decode=24, max_ctx=300, n_roots=3)
    tens = W.make_tensors(W.TINY, batch, 21)
    y, _ = check_step(lib, W.TINY, batch, tens)
    e, src = W.expand_batch(batch)
    te = W.make_tensors(W.TINY, batch, 21)
    te.k_pool = tens.k_pool[np.maximum(src, 0)]
    te.v_pool = tens.v_pool[np.maximum(src, 0)]
    y2, _, _, _ = run_step(lib, W.TINY, e, te)
    # same math, different grouping of the softmax partials: equal up to bf16 rounding of the output
    assert np.max(np.abs(y - y2)) / np.max(np.abs(y)) < 1e-2
    assert np.mean(np.abs(y - y2)) < MAE


def test_layers_back_to_back(lib):
    # three layers with their own weights and pools behind one descriptor; the activations passed
    # between layers are bf16 (that is the boundary's dtype), so the oracle chain rounds them too
    import dataclasses
    import torch
    shape = W.TINY
    batch = W.batch_random(11, n_prefill=3, n_decode=12, max_q=50, max_ctx=300)
    tens = [W.make_tensors(shape, batch, 20 + l, gains="random") for l in range(3)]
    layer = lib.Layer(shape, device=0)
    devs = [layer.upload(t, batch) for t in tens]
    y = layer.blend_layers(devs, batch)
    torch.cuda.synchronize()
    x = xd = tens[0].x
    for l, t in enumerate(tens):
        ref = O.layer_step(shape, dataclasses.replace(t, x=x), batch)
        diag = O.layer_step(shape, dataclasses.replace(t, x=xd), batch, storage="bf16")
        x = W.round_to_bf16(ref["y"].astype(np.float32))
        xd = diag["y"].astype(np.float32)
        k, v = layer.unpack_pool(devs[l].kv_pool, devs[l].n_pages)
        kn = to_np(k)[ref["dest"][:, 0], ref["dest"][:, 1]]
        assert errs(kn, ref["k_new"])[0] <= MAXREL, "layer %d keys" % l
    check(to_np(y), ref["y"], diag["y"], "3 layers")
    # one layer through the same entry point equals the single-step call bit for bit
    y1 = layer.blend_layers([layer.upload(tens[0], batch)], batch)
    y0 = layer.blend_step(layer.upload(tens[0], batch), batch)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)


@pytest.mark.parametrize("shape,n_layers", [(W.TINY, 4), (W.LayerShape(512, 8, 2, 128, 1288), 3)])
@pytest.mark.parametrize("knobs", [
    dict(head_cus_min=8, tail_workgroups=16, close_margin=2, ride_percent=100),
    dict(head_cus_min=48, tail_workgroups=208, close_margin=8, ride_percent=-1, attention_waves=4),
    dict(head_cus_min=0, tail_workgroups=24, close_margin=0, ride_percent=60),
])
def test_pipelined_layers_match_the_oracle_chain(lib, shape, n_layers, knobs):
    # BS_FLAG_PIPELINE: the decode rows run one stage ahead of the prefill rows across the layer
    # boundary, and the prefill rows' down projection of layer l carries decode attention of
    # layer l+1.  Every layer's appended keys and values and the final output against the oracle
    # chain (activations between layers are bf16, so the chain rounds them too).
    import dataclasses
    import torch
    rng = np.random.default_rng(31)
    seqs = [(130, 130, -1), (70, 200, -1), (45, 45, -1)] + [(1, 40 + 37 * i, -1) for i in range(40)]
    batch = W.assemble_batch(16, seqs, 3, [], rng)
    tens = [W.make_tensors(shape, batch, 40 + l, gains="random") for l in range(n_layers)]
    layer = lib.Layer(shape, device=0)
    layer.set_overlap(always=1, min_prefill_rows=1, **knobs)
    devs = [layer.upload(t, batch) for t in tens]
    layer.profile(True)
    y = layer.blend_layers(devs, batch, flags=lib.FLAG_OVERLAP | lib.FLAG_PIPELINE)
    torch.cuda.synchronize()
    prof = layer.profile_read()
    # the path was taken: the decode rows' GEMMs ran apart in every layer, and n_layers - 1 down
    # projections of the prefill rows were launches of their own
    assert prof["gemm_decode_rows"][1] > 0 and prof["gemm_down"][1] == n_layers
    x = xd = tens[0].x
    for l, t in enumerate(tens):
        ref = O.layer_step(shape, dataclasses.replace(t, x=x), batch)
        diag = O.layer_step(shape, dataclasses.replace(t, x=xd), batch, storage="bf16")
        x = W.round_to_bf16(ref["y"].astype(np.float32))
        xd = diag["y"].astype(np.float32)
        k, v = layer.unpack_pool(devs[l].kv_pool, devs[l].n_pages)
        k, v = to_np(k), to_np(v)
        assert errs(k[ref["dest"][:, 0], ref["dest"][:, 1]], ref["k_new"])[0] <= MAXREL, "layer %d keys" % l
        assert errs(v[ref["dest"][:, 0], ref["dest"][:, 1]], ref["v_new"])[0] <= MAXREL, "layer %d values" % l
        k0 = W.bf16_bits_to_f32(t.k_pool).astype(np.float64)
        written = np.zeros(k0.shape[:2], dtype=bool)
        written[ref["dest"][:, 0], ref["dest"][:, 1]] = True
        assert np.array_equal(k[~written], k0[~written]), "layer %d: a slot outside the append destinations changed" % l
    check(to_np(y), ref["y"], diag["y"], "%d pipelined layers" % n_layers)
    # and against the same layers co-scheduled one after the other (different tile shapes at most)
    devs2 = [layer.upload(t, batch) for t in tens]
    y2 = layer.blend_layers(devs2, batch, flags=lib.FLAG_OVERLAP)
    torch.cuda.synchronize()
    assert errs(to_np(y), to_np(y2))[0] <= MAXREL


def run_coscheduled(lib, shape, batch, tens, knobs, chunk_pages=0):
    import torch
    layer = lib.Layer(shape, device=0)
    layer.set_overlap(**knobs)
    if chunk_pages:
        layer.set_chunk_pages(chunk_pages)
    dev = layer.upload(tens, batch)
    layer.profile(True)
    y = layer.blend_step(dev, batch, flags=lib.FLAG_OVERLAP)
    torch.cuda.synchronize()
    run_coscheduled.taken = layer.profile_read()["gemm_decode_rows"][1] > 0   # the decode rows' GEMMs ran apart
    k, v = layer.unpack_pool(dev.kv_pool, dev.n_pages)
    return to_np(y), to_np(k), to_np(v)


@pytest.mark.parametrize("shape", [W.TINY, W.LayerShape(512, 8, 2, 128, 1288)])
@pytest.mark.parametrize("knobs", [
    dict(head_cus_min=8, tail_workgroups=16, close_margin=2, ride_percent=100),
    dict(head_cus_min=0, tail_workgroups=24, close_margin=0, ride_percent=60),
    dict(head_cus_min=16, tail_workgroups=0, close_margin=256, ride_percent=100, drain_in_last=0),
    dict(head_cus_min=48, tail_workgroups=208, close_margin=8, ride_percent=-1, attention_waves=4),
    dict(head_cus_min=8, tail_workgroups=8, close_margin=1, ride_percent=80, carry_down=0),
    dict(head_cus_min=8, tail_workgroups=8, close_margin=1, ride_percent=0)])
def test_coscheduled_step_matches_the_oracle(lib, shape, knobs):
    # decode attention of the 16-row units inside the prefill rows' GEMM launches: attention
    # workgroups ahead of the tiles only, behind them only, both; a queue that closes at once
    # (margin beyond the tile count) with everything left to a launch of its own; all units,
    # some or none of them waiting for the carrying launches; two or three carrying launches;
    # several chunks per tail, so the queue is longer than the workers are many
    knobs = dict(knobs, min_prefill_rows=1, always=1)
    batch = W.batch_random(17, n_prefill=4, n_decode=60, max_q=150, max_ctx=700, n_roots=3)
    tens = W.make_tensors(shape, batch, 17, gains="random")
    ref = O.layer_step(shape, tens, batch)
    diag = O.layer_step(shape, tens, batch, storage="bf16")
    y, k, v = run_coscheduled(lib, shape, batch, tens, knobs, chunk_pages=4)
    assert run_coscheduled.taken, "the step did not take the co-scheduled path"
    check(y, ref["y"], diag["y"], "co-scheduled %s" % knobs)
    kn = k[ref["dest"][:, 0], ref["dest"][:, 1]]
    assert errs(kn, ref["k_new"])[0] <= MAXREL


def test_coscheduled_step_agrees_with_the_serial_one(lib):
    # same arithmetic per output element; the GEMM tile shapes differ (the carrying launches use the
    # eight-wavefront tiles), so the fp32 sums may round differently: equal to within a bf16 step
    batch = W.batch_random(4, n_prefill=4, n_decode=30, max_q=120, max_ctx=500)
    tens = W.make_tensors(W.TINY, batch, 4)
    y0, _, _, _ = run_step(lib, W.TINY, batch, tens, 0)
    y1, _, _ = run_coscheduled(lib, W.TINY, batch, tens, dict(head_cus_min=8, tail_workgroups=16, min_prefill_rows=1, always=1))
    assert np.max(np.abs(y0 - y1)) <= 2.0 ** -7 * np.max(np.abs(y0))
    assert np.mean(np.abs(y0 - y1)) <= 1e-4


def test_coscheduled_flag_falls_back_where_nothing_can_overlap(lib):
    # no prefill rows, or no decode rows: the flag changes nothing
    for batch in (W.batch_decode_only(33, 130, seed=2), W.batch_prefill_only(3, 75, seed=2)):
        tens = W.make_tensors(W.TINY, batch, 2)
        y0, _, _, _ = run_step(lib, W.TINY, batch, tens, 0)
        y1, _, _ = run_coscheduled(lib, W.TINY, batch, tens, dict(head_cus_min=8, tail_workgroups=16, min_prefill_rows=1, always=1))
        assert not run_coscheduled.taken
        assert np.array_equal(y0, y1)


def test_cost_model_keeps_small_steps_serial(lib):
    # without `always` a tiny step is not expected to gain anything and runs the serial schedule
    batch = W.batch_random(4, n_prefill=4, n_decode=30, max_q=120, max_ctx=500)
    tens = W.make_tensors(W.TINY, batch, 4)
    y0, _, _, _ = run_step(lib, W.TINY, batch, tens, 0)
    y1, _, _ = run_coscheduled(lib, W.TINY, batch, tens, dict(min_prefill_rows=1))
    assert not run_coscheduled.taken and np.array_equal(y0, y1)


def test_repeated_calls_and_growing_workspace(lib):
    import torch
    layer = lib.Layer(W.TINY, device=0)
    for seed, (npf, ndec) in enumerate([(1, 4), (3, 40), (2, 9)]):
        batch = W.batch_random(30 + seed, n_prefill=npf, n_decode=ndec, max_q=200, max_ctx=300)
        tens = W.make_tensors(W.TINY, batch, seed)
        dev = layer.upload(tens, batch)
        y = layer.blend_step(dev, batch)
        torch.cuda.synchronize()
        ref = O.layer_step(W.TINY, tens, batch)["y"]
        maxrel, mae = errs(to_np(y), ref)
        assert maxrel <= MAXREL and mae <= MAE


def test_malformed_batch_is_an_error_code_on_the_gpu_path(lib):
    batch = W.batch_tiny(0)
    tens = W.make_tensors(W.TINY, batch, 0)
    layer = lib.Layer(W.TINY, device=0)
    dev = layer.upload(tens, batch)
    bad = batch.copy()
    bad.page_ids[0] = batch.n_pages + 5
    with pytest.raises(lib.BlendStepError) as ei:
        layer.blend_step(dev, bad)
    assert ei.value.code == -1
    # the context still works afterwards
    y = layer.blend_step(dev, batch)
    assert np.isfinite(to_np(y)).all()


def test_builder_batch_through_the_layer(lib):
    # host builder -> descriptor -> blended step, against the layer oracle on the same descriptor
    from paper_2411_16102_amd import binding
    rng = np.random.default_rng(5)
    b = binding.Builder(8_030_000_000, 131072, 2.5e15, 8.0e12, 600_000_000, 16)
    for g in range(3):
        prefix = [int(t) for t in rng.integers(0, 1000, int(rng.integers(40, 120)))]
        for _ in range(6):
            toks = prefix + [int(t) for t in rng.integers(0, 1000, int(rng.integers(1, 30)))]
            b.add(toks, int(rng.integers(50, 600)), len(toks) + int(rng.integers(0, 100)))
    for _ in range(4):
        b.add([int(t) for t in rng.integers(0, 1000, int(rng.integers(20, 90)))], 4, 0)
    b.finalize()
    info, d = b.next_batch(prefill_budget=128)
    assert info["n_prefill"] > 0 and info["n_decode"] > 0 and d["n_nodes"] > 0
    batch = W.Batch(page_size=16, n_seq=d["n_seq"], n_prefill=d["n_prefill"], n_rows=d["n_rows"],
                    row_start=d["row_start"], kv_len=d["kv_len"], page_start=d["page_start"], page_ids=d["page_ids"],
                    n_nodes=d["n_nodes"], node_parent=d["node_parent"], node_page_start=d["node_page_start"],
                    node_page_ids=d["node_page_ids"], node_seq_first=d["node_seq_first"],
                    node_seq_count=d["node_seq_count"], seq_leaf_node=d["seq_leaf_node"], n_pages=d["n_pages"] + 3)
    tens = W.make_tensors(W.TINY, batch, 5)
    check_step(lib, W.TINY, batch, tens)
