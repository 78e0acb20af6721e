"""CPU-side checks of the library: exported symbols, descriptor validation and
bit-exact page resolution against the oracle's resolver.  No GPU is touched."""
import numpy as np
import pytest

from oracle import layer as O
from paper_2411_16102_amd import binding, workloads as W


@pytest.fixture(scope="module")
def host_layer():
    return binding.Layer(W.TINY, device=-1)


def test_library_exports_every_declared_function():
    names = binding.declared_functions()
    assert "bs_blend_step" in names and "bs_create" in names and len(names) >= 15
    assert binding.check_symbols()


def test_gpu_entry_points_refuse_a_host_only_context(host_layer):
    b = W.batch_tiny()
    d, keep = binding.marshal_batch(b)
    import ctypes as C
    w = binding.Weights(*[C.c_void_p(8)] * 6)
    rc = host_layer.lib.bs_blend_step(host_layer.h, C.byref(w), C.byref(d), C.c_void_p(8), C.c_void_p(16),
                                      C.c_void_p(24), b.n_pages, None, 0)
    assert rc == -1 and "host-only" in host_layer.last_error()


@pytest.mark.parametrize("name", list(W.CONFIGS))
def test_generated_configs_validate(host_layer, name):
    shape, fn = W.CONFIGS[name]
    b = fn()
    lay = binding.Layer(shape, device=-1)
    assert lay.validate(b) == 0, lay.last_error()


@pytest.mark.parametrize("seed", range(6))
def test_row_resolution_is_bit_exact(host_layer, seed):
    b = W.batch_random(seed, n_prefill=4, n_decode=12, max_q=70, max_ctx=300)
    pg, sl = host_layer.resolve_rows(b)
    row = 0
    for s in range(b.n_seq):
        q = int(b.row_start[s + 1] - b.row_start[s])
        for j in range(q):
            want = O.resolve(b, s, int(b.kv_len[s]) - q + j)
            assert (int(pg[row]), int(sl[row])) == want
            row += 1
    assert row == b.n_rows


def test_row_resolution_full_size_config(host_layer):
    shape, fn = W.CONFIGS["blended_8b"]
    b = fn()
    lay = binding.Layer(shape, device=-1)
    pg, sl = lay.resolve_rows(b)
    rng = np.random.default_rng(0)
    row_seq = np.repeat(np.arange(b.n_seq), b.q_len())
    for r in rng.integers(0, b.n_rows, 300):
        s = int(row_seq[r])
        pos = int(b.kv_len[s]) - int(b.row_start[s + 1] - b.row_start[s]) + int(r - b.row_start[s])
        assert (int(pg[r]), int(sl[r])) == O.resolve(b, s, pos)


def _bad(host_layer, b, n_pages=None):
    rc = host_layer.validate(b, n_pages)
    return rc, host_layer.last_error()


def test_malformed_descriptors_are_error_codes(host_layer):
    good = W.batch_random(1, n_prefill=2, n_decode=8)
    assert host_layer.validate(good) == 0

    b = good.copy(); b.page_ids[3] = good.n_pages
    rc, msg = _bad(host_layer, b); assert rc == -1 and "outside the pool" in msg

    b = good.copy(); b.page_ids[0] = -1
    assert _bad(host_layer, b)[0] == -1

    b = good.copy(); b.kv_len[0] = int(np.diff(b.page_start)[0]) * 16 + 1
    rc, msg = _bad(host_layer, b); assert rc == -1 and "exceeds its" in msg

    b = good.copy(); b.row_start[1] = b.row_start[0]
    assert _bad(host_layer, b)[0] == -1

    b = good.copy(); b.n_rows += 1
    assert _bad(host_layer, b)[0] == -1

    b = good.copy(); b.page_start[2] = b.page_start[1] - 1
    assert _bad(host_layer, b)[0] == -1

    b = good.copy(); b.kv_len[b.n_prefill] = 0
    assert _bad(host_layer, b)[0] == -1

    # a decode sequence with two rows
    b = good.copy(); b.n_prefill = 0
    assert _bad(host_layer, b)[0] == -1

    # kv_len beyond the RoPE table
    b = W.assemble_batch(16, [(1, 20000, -1)], 0, [], None)
    rc, msg = _bad(host_layer, b); assert rc == -1 and "max_positions" in msg


def test_shared_page_may_not_be_written(host_layer):
    # two sequences whose last (written) page is the same physical page
    b = W.assemble_batch(16, [(1, 20, -1), (1, 20, -1)], 0, [], None)
    b.page_ids[3] = b.page_ids[1]
    rc, msg = _bad(host_layer, b)
    assert rc == -1 and "more than once" in msg
    # a node page may not be written even by its only member
    b = W.assemble_batch(16, [(1, 33, 0)], 0, [(-1, 2)], None)
    assert host_layer.validate(b) == 0
    b.kv_len[0] = 32
    rc, msg = _bad(host_layer, b)
    assert rc == -1


def test_inconsistent_nodes_are_rejected(host_layer):
    good = W.batch_tiny()
    assert host_layer.validate(good) == 0
    b = good.copy(); b.node_page_ids[2] = (b.node_page_ids[2] + 1) % good.n_pages
    rc, msg = _bad(host_layer, b); assert rc == -1 and "does not carry" in msg
    b = good.copy(); b.node_seq_count[0] = 7
    assert _bad(host_layer, b)[0] == -1
    b = good.copy(); b.node_seq_first[0] = 1   # run would include a prefill segment
    assert _bad(host_layer, b)[0] == -1
    b = good.copy(); b.seq_leaf_node[0] = 0    # prefill segment as a node member
    assert _bad(host_layer, b)[0] == -1
    b = good.copy(); b.node_parent[0] = 0
    assert _bad(host_layer, b)[0] == -1
    b = good.copy(); b.seq_leaf_node[5] = 3
    assert _bad(host_layer, b)[0] == -1


def test_empty_batch_is_valid(host_layer):
    b = W.assemble_batch(16, [], 0, [], None)
    assert host_layer.validate(b) == 0


def test_tuning_knobs_reject_values_outside_their_range(host_layer):
    for bad in (0, 1, 3, 66, -2):
        assert host_layer.lib.bs_set_chunk_pages(host_layer.h, bad) == -1 and "chunk_pages" in host_layer.last_error()
    for ok in (2, 32, 64):
        assert host_layer.lib.bs_set_chunk_pages(host_layer.h, ok) == 0
    assert host_layer.lib.bs_set_gemm_tiles(host_layer.h, 4) == -1
    assert host_layer.lib.bs_set_gemm_tiles(host_layer.h, 7) == -1
    assert host_layer.lib.bs_set_gemm_tiles(host_layer.h, 0) == 0
    good = host_layer.get_overlap()
    for bad in (dict(head_cus_min=4), dict(head_cus_min=200), dict(head_cus_min=-8), dict(tail_workgroups=257),
                dict(close_margin=-1), dict(min_prefill_rows=0), dict(ride_percent=101), dict(ride_percent=-2),
                dict(attention_waves=0), dict(attention_waves=9), dict(head_cus_max=7), dict(head_cus_max=200)):
        with pytest.raises(binding.BlendStepError):
            host_layer.set_overlap(**bad)
    assert host_layer.get_overlap() == good
    host_layer.set_overlap(head_cus_min=48, ride_percent=50)
    assert host_layer.get_overlap()["head_cus_min"] == 48 and host_layer.get_overlap()["ride_percent"] == 50
    host_layer.set_overlap(**good)
