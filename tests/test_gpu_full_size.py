"""Parity at the full sizes of the benchmark configurations, in both schedules bench.py may time.

decode_8b, prefill_8b, blended_8b: EVERY element of y against the exact oracle (the oracle needs
5 to 40 s per configuration on the machine's host cores).  blended_70b (8.9 TFLOP in float64): rows
sampled so that every block of 256 consecutive rows (the tallest GEMM tile) and every prefill
segment at several depths is covered, within about a minute of oracle time.  At every size the KV
append is checked too: exactly the destination slots of the pool change (compared on the device,
bit for bit, against the uploaded pool), page and slot of every row match the oracle's resolver,
and the appended keys and values match the oracle's.

Tolerance: the one rule of tests/parity_rule.py; every figure is printed.
"""
import numpy as np
import pytest

from oracle import layer as O
from paper_2411_16102_amd import workloads as W
from parity_rule import MAXREL, check, errs

pytestmark = pytest.mark.gpu


def rows_covering_every_block(batch, rng, block=256, per_block=3):
    rows = set()
    for s in range(batch.n_prefill):       # first, middle and last row of every prefill segment
        r0, r1 = int(batch.row_start[s]), int(batch.row_start[s + 1])
        rows |= {r0, (r0 + r1) // 2, r1 - 1}
    for b0 in range(0, batch.n_rows, block):
        b1 = min(batch.n_rows, b0 + block)
        rows |= {int(r) for r in rng.integers(b0, b1, per_block)} | {b0, b1 - 1}
    n_dec = batch.n_seq - batch.n_prefill
    if n_dec:                               # the shortest and the longest decode context
        kv = batch.kv_len[batch.n_prefill:]
        rows |= {int(batch.row_start[batch.n_prefill + int(np.argmin(kv))]),
                 int(batch.row_start[batch.n_prefill + int(np.argmax(kv))])}
    return sorted(rows)


@pytest.mark.parametrize("name", ["decode_8b", "prefill_8b", "blended_8b", "blended_70b"])
def test_full_size_config(lib, name):
    import torch
    shape, make = W.CONFIGS[name]
    batch = make(seed=0)
    tens = W.make_tensors(shape, batch, 0)
    layer = lib.Layer(shape, device=0)
    rows = None if name != "blended_70b" else rows_covering_every_block(batch, np.random.default_rng(123))
    sel = slice(None) if rows is None else rows
    print("%s: oracle on %s rows" % (name, "all %d" % batch.n_rows if rows is None else "%d of %d" % (len(rows), batch.n_rows)), flush=True)
    ref = O.layer_step(shape, tens, batch, rows=rows)
    diag = O.layer_step(shape, tens, batch, rows=rows, storage="bf16")
    pg, sl = layer.resolve_rows(batch)
    assert np.array_equal(pg, ref["dest"][:, 0]) and np.array_equal(sl, ref["dest"][:, 1])
    # the rows whose keys and values the oracle has computed (all rows of the sampled sequences)
    have_kv = np.nonzero(~np.isnan(ref["k_new"][:, 0, 0]))[0]
    dest = torch.from_numpy(ref["dest"].astype(np.int64)).cuda()
    for flags in (0, 1):
        dev = layer.upload(tens, batch)                       # a fresh pool for each schedule
        pool0 = dev.kv_pool.clone()
        y = layer.blend_step(dev, batch, flags=flags)
        torch.cuda.synchronize()
        got = y.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        check(got[sel], ref["y"][sel], diag["y"][sel], "%s flags=%d y" % (name, flags))
        # KV append, on the device: which (page, slot) pairs of the pool differ from the uploaded one
        k1, v1 = layer.unpack_pool(dev.kv_pool, dev.n_pages)
        k0, v0 = layer.unpack_pool(pool0, dev.n_pages)
        changed = ((k1.view(torch.int16) != k0.view(torch.int16)).any(dim=3).any(dim=2) |
                   (v1.view(torch.int16) != v0.view(torch.int16)).any(dim=3).any(dim=2))
        allowed = torch.zeros_like(changed)
        allowed[dest[:, 0], dest[:, 1]] = True
        assert not bool((changed & ~allowed).any()), "a slot outside the append destinations changed"
        assert int(changed.sum()) == batch.n_rows, "not every destination slot was written"
        d = dest[torch.from_numpy(have_kv).cuda()]
        kn = k1[d[:, 0], d[:, 1]].float().cpu().numpy().astype(np.float64)
        vn = v1[d[:, 0], d[:, 1]].float().cpu().numpy().astype(np.float64)
        check(kn, ref["k_new"][have_kv], diag["k_new"][have_kv], "%s flags=%d appended keys" % (name, flags))
        check(vn, ref["v_new"][have_kv], diag["v_new"][have_kv], "%s flags=%d appended values" % (name, flags))
        del k1, v1, k0, v0, pool0, dev


def test_full_size_two_pipelined_layers(lib):
    """blended_8b through two layers with the parts of the batch pipelined across the layer boundary
    (the down projection of the first layer's prefill rows carries decode attention of the second): the
    second layer's output, every element, and its KV append against the oracle chain."""
    import dataclasses
    import torch
    shape, make = W.CONFIGS["blended_8b"]
    batch = make(seed=0)
    tens = [W.make_tensors(shape, batch, l) for l in range(2)]
    layer = lib.Layer(shape, device=0)
    layer.set_overlap(always=1)
    devs = [layer.upload(t, batch) for t in tens]
    layer.profile(True)
    y = layer.blend_layers(devs, batch, flags=lib.FLAG_OVERLAP | lib.FLAG_PIPELINE)
    torch.cuda.synchronize()
    prof = layer.profile_read()
    assert prof["gemm_decode_rows"][1] > 0 and prof["gemm_down"][1] == 2    # the pipelined path ran
    got = y.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    print("oracle: layer 1 of 2", flush=True)
    ref1 = O.layer_step(shape, tens[0], batch)
    diag1 = O.layer_step(shape, tens[0], batch, storage="bf16")
    x2 = W.round_to_bf16(ref1["y"].astype(np.float32))     # the activations between layers are bf16
    print("oracle: layer 2 of 2", flush=True)
    ref2 = O.layer_step(shape, dataclasses.replace(tens[1], x=x2), batch)
    # the storage error of two layers: the diagnostic chain carries its own first-layer output
    diag2 = O.layer_step(shape, dataclasses.replace(tens[1], x=diag1["y"].astype(np.float32)), batch, storage="bf16")
    check(got, ref2["y"], diag2["y"], "two pipelined layers, y")
    for l, ref in ((0, ref1), (1, ref2)):
        k1, v1 = layer.unpack_pool(devs[l].kv_pool, devs[l].n_pages)
        dest = torch.from_numpy(ref["dest"].astype(np.int64)).cuda()
        kn = k1[dest[:, 0], dest[:, 1]].float().cpu().numpy().astype(np.float64)
        vn = v1[dest[:, 0], dest[:, 1]].float().cpu().numpy().astype(np.float64)
        assert errs(kn, ref["k_new"])[0] <= MAXREL and errs(vn, ref["v_new"])[0] <= MAXREL, "layer %d KV append" % l
        del k1, v1
