"""The entry point that allocates nothing (bs_attention_noalloc) against bs_attention: same kernels,
same descriptor, so the outputs must be equal bit for bit; two calls in a row on one context, the
second with a smaller batch (the scratch array keeps the first call's contents), then a batch beyond
the stated limits, which must be refused before anything is enqueued."""
import numpy as np
import pytest

from paper_2411_16102_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_noalloc_attention_matches_the_allocating_entry_point(lib):
    import torch
    shape = W.LayerShape(512, 8, 2, 128, 256)
    layer = lib.Layer(shape, device=0)
    layer.set_chunk_pages(4)
    for seed, (n_pre, n_dec, ctx) in enumerate([(4, 48, 900), (2, 9, 200)]):
        batch = W.batch_random(40 + seed, n_prefill=n_pre, n_decode=n_dec, max_q=120, max_ctx=ctx, n_roots=3)
        tens = W.make_tensors(shape, batch, seed)
        rng = np.random.default_rng(seed)
        q = W.round_to_bf16(rng.standard_normal((batch.n_rows, shape.n_q_heads * shape.head_dim), dtype=np.float32))
        tq = torch.from_numpy(q).cuda().to(torch.bfloat16)
        pool = layer.pack_pool(tens.k_pool, tens.v_pool)
        ref = layer.attention(batch, tq, pool, batch.n_pages)
        out = torch.zeros_like(tq)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]   # the driver's figure: sees the library's own allocations too
        layer.attention_noalloc(batch, tq, pool, batch.n_pages, out)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before
        assert torch.equal(out, ref), "call %d differs from bs_attention" % seed
        assert bool(torch.isfinite(out.float()).all())


def test_noalloc_attention_refuses_what_does_not_fit(lib):
    import torch
    # 8B heads: one partial state is 32 x 130 floats = 16.6 KB, so 15 MiB hold 945 of them; 1200 decode
    # sequences need 1200
    shape = W.LayerShape(512, 32, 8, 128, 256)
    layer = lib.Layer(shape, device=0)
    batch = W.batch_decode_only(1200, 40, seed=1)
    tens = W.make_tensors(shape, batch, 1)
    pool = layer.pack_pool(tens.k_pool, tens.v_pool)
    q = torch.zeros((batch.n_rows, shape.n_q_heads * shape.head_dim), dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 3.0)
    with pytest.raises(lib.BlendStepError) as ei:
        layer.attention_noalloc(batch, q, pool, batch.n_pages, out)
    assert ei.value.code == -1 and "exceed the limit" in str(ei.value)
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
    # the allocating entry point takes the same batch
    assert bool(torch.isfinite(layer.attention(batch, q, pool, batch.n_pages).float()).all())
