"""CPU oracle for one blended step of a Llama-style decoder layer.

TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition that the HIP path
is checked against; nothing on the product path may import it.  It shares no
code with the GPU library and takes every input as a numpy array.

What it computes.  BlendServe (Section 2.1) describes the layer only in words:
Q/K/V projections, softmax attention in which several query heads attend to one
key/value head (GQA), a feed-forward network, a KV cache that a decode step
re-reads in full, and (Section 4.2) "small operators": normalisation, activation
and position embedding.  Prefix sharing and request reordering are lossless
(Sections 2.2, 3.3), so the reference result is the plain layer evaluated per
sequence over that sequence's own, physically unshared ("expanded") KV:

    h  = rmsnorm(x; g_attn);  q,k,v = h W_q, h W_k, h W_v;  q,k <- rope(., pos)
    K_i, V_i = [cached tokens of sequence i gathered through its page table ;
                this step's k, v of sequence i]
    o  = softmax(q K_i^T / sqrt(dh) + causal mask) V_i        (two-pass softmax)
    x1 = x + o W_o;  h2 = rmsnorm(x1; g_ffn)
    y  = x1 + (silu(h2 W_gate) * (h2 W_up)) W_down

The Llama-style choices the paper leaves open (pre-norm RMSNorm with fp mean of
squares over d and eps inside the root; rotate-half RoPE pairing (i, i+dh/2)
with angle pos * theta^(-2i/dh); scale 1/sqrt(dh); silu(z) = z / (1 + exp(-z));
K cached after RoPE) are fields of the shape or stated where they are used.

Arithmetic is float64 throughout (numpy matmul is the one library step): the
inputs are bfloat16 values, and in float64 the sums of up to 28672 products are
exact to 1e-13 of their size, so what a comparison against this oracle shows is
the error of the path under test alone.  A float32 oracle would add an error of
its own of about 1e-5 relative, and its matmul would have to be blocked to run at
all at the full sizes; float64 is the stricter reference and the plainer code.
Parity is claimed against this exact mode only.

storage="bf16" is a DIAGNOSTIC, not a reference: it rounds to bfloat16 every
tensor that a plain bfloat16 layer writes to memory between two operators, in
the textbook order (the normalised activations h and h2, q, k, v, the softmax
probabilities as operand of their product with V, the attention output, x1, the
SwiGLU output, y), whatever a particular kernel pipeline keeps wider.  Its distance from the exact mode shows how much error bfloat16 storage
alone puts into the output at a given shape; no test gates on it.

Pins (tests/test_oracle_layer.py): brute-force dense masked attention in pure
Python on tiny inputs; closed forms for RMSNorm, RoPE and SwiGLU; kv_len = 1,
equal-keys and dominant-logit special cases; shared-vs-expanded, request-order
and chunking invariants; page resolution through a planted-key property.
"""
from __future__ import annotations

import numpy as np


# -- bfloat16 storage rounding (own copy: the oracle stands alone) -------------
def _store_bf16(a: np.ndarray) -> np.ndarray:
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32)
    r = (u + (((u >> 16) & 1) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def _bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _as_f64_pool(pool: np.ndarray) -> np.ndarray:
    return _bits_to_f64(pool) if pool.dtype == np.uint16 else np.asarray(pool, dtype=np.float64)


# -- small operators ------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def rope(v: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate-half position embedding.  v: [n, heads, dh], pos: [n].

    Pair (i, i + dh/2) of every head is rotated by the angle pos * theta^(-2i/dh).
    """
    v = np.asarray(v, dtype=np.float64)
    dh = v.shape[-1]
    half = dh // 2
    i = np.arange(half, dtype=np.float64)
    freq = np.power(float(theta), -2.0 * i / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * freq[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


# -- paged KV -------------------------------------------------------------------
def resolve(batch, s: int, t: int):
    """(physical page, slot) of token t of sequence s."""
    ps = batch.page_size
    return int(batch.page_ids[int(batch.page_start[s]) + t // ps]), t % ps


def gather_kv(batch, s: int, n_tokens: int, k_pool: np.ndarray, v_pool: np.ndarray):
    """Private (expanded) copy of the first n_tokens cached tokens of sequence s:
    K, V of shape [n_tokens, Hkv, dh] in float64."""
    ps = batch.page_size
    n_pg = -(-n_tokens // ps)
    ids = batch.page_ids[int(batch.page_start[s]):int(batch.page_start[s]) + n_pg].astype(np.int64)
    hkv, dh = k_pool.shape[2], k_pool.shape[3]
    K = _as_f64_pool(k_pool[ids]).reshape(n_pg * ps, hkv, dh)[:n_tokens]
    V = _as_f64_pool(v_pool[ids]).reshape(n_pg * ps, hkv, dh)[:n_tokens]
    return K, V


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, first_pos: int, storage: str = "exact") -> np.ndarray:
    """Exact softmax attention of n query rows over one sequence's keys.

    q: [n, Hq, dh]; K, V: [L, Hkv, dh] with L = first_pos + n.  Row j sits at
    position first_pos + j and sees keys 0 .. first_pos + j.  Query head h reads
    key/value head h // (Hq / Hkv).  Two passes: row maximum, then exp and sum.
    storage="bf16" (diagnostic, see the module header): the probabilities are rounded to
    bfloat16 where they become the operand of the product with V, as in any bfloat16
    attention; the row sums keep the unrounded values.
    """
    n, hq, dh = q.shape
    L, hkv, _ = K.shape
    assert L == first_pos + n
    grp = hq // hkv
    out = np.empty((n, hq, dh), dtype=np.float64)
    scale = 1.0 / np.sqrt(float(dh))
    visible = np.arange(L)[None, :] <= (first_pos + np.arange(n))[:, None]
    for h in range(hq):
        kh = h // grp
        s = (q[:, h, :] @ K[:, kh, :].T) * scale
        s = np.where(visible, s, -np.inf)
        m = np.max(s, axis=1, keepdims=True)
        p = np.exp(s - m)
        pv = _store_bf16(p) if storage == "bf16" else p
        out[:, h, :] = (pv @ V[:, kh, :]) / np.sum(p, axis=1, keepdims=True)
    return out


# -- the layer --------------------------------------------------------------------
def layer_step(shape, tensors, batch, rows=None, storage: str = "exact"):
    """One blended step.  Returns a dict with

      y        [T, d]        layer output (rows not asked for are NaN)
      k_new    [T, Hkv, dh]  this step's keys after RoPE   (NaN where not computed)
      v_new    [T, Hkv, dh]  this step's values
      dest     [T, 2] int32  (physical page, slot) each row's k, v are appended to
      attn     [T, Hq*dh]    attention output before the output projection
      x1       [T, d]        after the first residual add

    rows: optional list of row indices; only those rows get y (their sequences'
    keys and values are still computed for every earlier row of the same
    sequence, which is all causal attention needs).
    """
    assert storage in ("exact", "bf16")
    st = _store_bf16 if storage == "bf16" else (lambda a: np.asarray(a, dtype=np.float64))
    d, hq, hkv, dh = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    T = batch.n_rows
    x = np.asarray(tensors.x, dtype=np.float64)
    w_qkv = np.asarray(tensors.w_qkv, dtype=np.float64)
    want = np.zeros(T, dtype=bool)
    if rows is None:
        want[:] = True
    else:
        want[np.asarray(rows, dtype=np.int64)] = True

    row_seq = np.repeat(np.arange(batch.n_seq), np.diff(batch.row_start))
    q_len = np.diff(batch.row_start).astype(np.int64)
    first_pos = batch.kv_len.astype(np.int64) - q_len
    pos = first_pos[row_seq] + (np.arange(T) - batch.row_start[row_seq])
    seq_wanted = np.zeros(batch.n_seq, dtype=bool)
    seq_wanted[row_seq[want]] = True
    need_qkv = seq_wanted[row_seq]

    y = np.full((T, d), np.nan)
    k_new = np.full((T, hkv, dh), np.nan)
    v_new = np.full((T, hkv, dh), np.nan)
    attn = np.full((T, hq * dh), np.nan)
    x1 = np.full((T, d), np.nan)
    dest = np.zeros((T, 2), dtype=np.int32)
    for r in range(T):
        dest[r] = resolve(batch, int(row_seq[r]), int(pos[r]))

    idx = np.nonzero(need_qkv)[0]
    qkv = st(rmsnorm(x[idx], tensors.g_attn, shape.rms_eps)) @ w_qkv
    q = rope(qkv[:, :hq * dh].reshape(-1, hq, dh), pos[idx], shape.rope_theta)
    k = rope(qkv[:, hq * dh:(hq + hkv) * dh].reshape(-1, hkv, dh), pos[idx], shape.rope_theta)
    v = qkv[:, (hq + hkv) * dh:].reshape(-1, hkv, dh)
    q_all = np.full((T, hq, dh), np.nan)
    q_all[idx] = st(q)
    k_new[idx] = st(k)
    v_new[idx] = st(v)

    for s in range(batch.n_seq):
        if not seq_wanted[s]:
            continue
        r0, r1 = int(batch.row_start[s]), int(batch.row_start[s + 1])
        c = int(first_pos[s])
        Kc, Vc = gather_kv(batch, s, c, tensors.k_pool, tensors.v_pool)
        K = np.concatenate([Kc, k_new[r0:r1]], axis=0)
        V = np.concatenate([Vc, v_new[r0:r1]], axis=0)
        sel = np.nonzero(want[r0:r1])[0]
        if len(sel) == r1 - r0:
            o = attention(q_all[r0:r1], K, V, c, storage)
            attn[r0:r1] = o.reshape(r1 - r0, hq * dh)
        else:
            for j in sel:  # one row at a time over its visible keys
                o = attention(q_all[r0 + j:r0 + j + 1], K[:c + j + 1], V[:c + j + 1], c + j, storage)
                attn[r0 + j] = o.reshape(hq * dh)

    w = np.nonzero(want)[0]
    a_in = st(attn[w])
    attn[w] = a_in
    x1w = st(x[w] + a_in @ np.asarray(tensors.w_o, dtype=np.float64))
    x1[w] = x1w
    h2 = st(rmsnorm(x1w, tensors.g_ffn, shape.rms_eps))
    gate = h2 @ np.asarray(tensors.w_gate, dtype=np.float64)
    up = h2 @ np.asarray(tensors.w_up, dtype=np.float64)
    act = st(silu(gate) * up)
    y[w] = st(x1w + act @ np.asarray(tensors.w_down, dtype=np.float64))
    return dict(y=y, k_new=k_new, v_new=v_new, dest=dest, attn=attn, x1=x1, q=q_all, pos=pos)


def append_kv(batch, result, k_pool: np.ndarray, v_pool: np.ndarray):
    """Pools (float64 copies) after this step's keys and values are written to
    their (page, slot) destinations."""
    kp = _as_f64_pool(k_pool).copy()
    vp = _as_f64_pool(v_pool).copy()
    for r in range(batch.n_rows):
        pg, sl = result["dest"][r]
        kp[pg, sl] = result["k_new"][r]
        vp[pg, sl] = result["v_new"][r]
    return kp, vp
