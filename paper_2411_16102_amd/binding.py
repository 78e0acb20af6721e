"""ctypes binding of libblendstep.so: argument marshalling only.

Every step of the layer runs inside the library's HIP kernels; PyTorch is used
here for device memory and the current stream.  If the shared object is missing
the import of the library fails loudly: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
import re
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SO = os.path.join(_HERE, "libblendstep.so")
_HEADERS = [os.path.join(_ROOT, "include", "blendstep.h"), os.path.join(_ROOT, "include", "blendstep_builder.h")]

_i32p = C.POINTER(C.c_int32)

K_NAMES = ["prep", "gemm_qkv", "attn_prefill", "attn_decode", "attn_merge", "gemm_o", "gemm_gate_up", "gemm_down",
           "attn_queue_rest", "gemm_decode_rows"]
FLAG_SERIAL, FLAG_OVERLAP, FLAG_PIPELINE = 0, 1, 2


class LayerCfg(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("page_size", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("max_positions", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_qkv", "w_o", "w_gate_up", "w_down", "g_attn", "g_ffn")]


class BatchDesc(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("n_prefill", C.c_int32), ("n_rows", C.c_int32),
                ("row_start", _i32p), ("kv_len", _i32p), ("page_start", _i32p), ("page_ids", _i32p),
                ("n_nodes", C.c_int32), ("node_parent", _i32p), ("node_page_start", _i32p),
                ("node_page_ids", _i32p), ("node_seq_first", _i32p), ("node_seq_count", _i32p),
                ("seq_leaf_node", _i32p)]


class OverlapKnobs(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("head_cus_min", "tail_workgroups", "close_margin", "min_prefill_rows",
                                         "ride_percent", "attention_waves", "carry_down", "drain_in_last", "head_cus_max", "always")]


class SplitInfo(C.Structure):
    _fields_ = [("n_split", C.c_int32), ("rounds", C.c_int32), ("monotone", C.c_int32),
                ("recompute_tokens", C.c_int64)]


class CostModel(C.Structure):
    _fields_ = [("p_model", C.c_int64), ("kv_bytes", C.c_int64), ("compute", C.c_double), ("bandwidth", C.c_double),
                ("mem_bytes", C.c_int64), ("page_size", C.c_int32)]


class ScanInfo(C.Structure):
    _fields_ = [("rho_rt", C.c_double), ("rho_l", C.c_double), ("rho_r", C.c_double), ("m_l", C.c_double),
                ("m_r", C.c_double), ("n_l", C.c_int64), ("n_r", C.c_int64), ("c_l", C.c_int64), ("c_r", C.c_int64),
                ("n_prefill", C.c_int32), ("n_decode", C.c_int32)]


class BatchOwned(C.Structure):
    _fields_ = [("batch", BatchDesc), ("seq_request", _i32p), ("n_pages", C.c_int64), ("info", ScanInfo)]


class SchedCfg(C.Structure):
    _fields_ = [("mem_tokens", C.c_int64), ("token_budget", C.c_int32), ("n_pages", C.c_int32),
                ("relocate_pct", C.c_int32), ("row_multiple", C.c_int32)]


class SchedStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("steps", "rows", "prefill_rows", "decode_rows", "prompt_tokens_skipped", "tokens_out",
                                         "finished", "peak_tokens", "peak_pages", "relocated", "mem_left", "mem_right")]


class BlendStepError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("blendstep error %d: %s" % (code, msg))
        self.code = code


def declared_functions():
    """Names of the functions the public headers declare."""
    names = []
    for h in _HEADERS:
        if not os.path.exists(h):
            continue
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names += re.findall(r"\b(bs_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


_lib = None


def raw():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise ImportError("%s is not built: run `python __graft_entry__.py` (hipcc, gfx950) first" % _SO)
        # PyTorch ships its own HIP runtime; load it first so that this library binds
        # to the same runtime instance (two runtimes in one process do not share a GPU)
        import torch  # noqa: F401
        lib = C.CDLL(_SO)
        lib.bs_create.argtypes = [C.POINTER(LayerCfg), C.c_int, C.POINTER(C.c_void_p)]
        lib.bs_destroy.argtypes = [C.c_void_p]
        lib.bs_destroy.restype = None
        lib.bs_last_error.argtypes = [C.c_void_p]
        lib.bs_last_error.restype = C.c_char_p
        lib.bs_kv_page_bytes.argtypes = [C.c_void_p]
        lib.bs_kv_page_bytes.restype = C.c_int64
        lib.bs_kv_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        lib.bs_kv_unpack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        lib.bs_blend_layers.argtypes = [C.c_void_p, C.c_int32, C.POINTER(Weights), C.POINTER(BatchDesc), C.c_void_p, C.c_void_p,
                                        C.POINTER(C.c_void_p), C.c_int64, C.c_void_p, C.c_uint32]
        lib.bs_blend_step.argtypes = [C.c_void_p, C.POINTER(Weights), C.POINTER(BatchDesc), C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_int64, C.c_void_p, C.c_uint32]
        lib.bs_validate_batch.argtypes = [C.c_void_p, C.POINTER(BatchDesc), C.c_int64]
        lib.bs_resolve_rows.argtypes = [C.c_void_p, C.POINTER(BatchDesc), _i32p, _i32p]
        lib.bs_profile_enable.argtypes = [C.c_void_p, C.c_int]
        lib.bs_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        lib.bs_profile_reset.argtypes = [C.c_void_p]
        lib.bs_set_chunk_pages.argtypes = [C.c_void_p, C.c_int32]
        lib.bs_set_gemm_tiles.argtypes = [C.c_void_p, C.c_int32]
        lib.bs_set_overlap.argtypes = [C.c_void_p, C.POINTER(OverlapKnobs)]
        lib.bs_get_overlap.argtypes = [C.c_void_p, C.POINTER(OverlapKnobs)]
        lib.bs_attention_noalloc.argtypes = [C.c_void_p, C.POINTER(BatchDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                             C.c_void_p]
        lib.bs_overlap_report.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        lib.bs_overlap_trace.argtypes = [C.c_void_p, C.c_int]
        lib.bs_overlap_trace_read.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_uint64), C.c_int64, C.POINTER(C.c_int64)]
        lib.bs_gemm_nt.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                   C.c_void_p]
        lib.bs_attention.argtypes = [C.c_void_p, C.POINTER(BatchDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                     C.c_void_p, C.c_uint32]
        _i64p = C.POINTER(C.c_int64)
        lib.bs_builder_create.argtypes = [C.POINTER(CostModel), C.POINTER(C.c_void_p)]
        lib.bs_builder_destroy.argtypes = [C.c_void_p]
        lib.bs_builder_destroy.restype = None
        lib.bs_builder_last_error.argtypes = [C.c_void_p]
        lib.bs_builder_last_error.restype = C.c_char_p
        lib.bs_builder_add.argtypes = [C.c_void_p, _i32p, C.c_int32, C.c_int32, C.c_int32]
        lib.bs_builder_finalize.argtypes = [C.c_void_p]
        lib.bs_builder_set_mem_model.argtypes = [C.c_void_p, C.c_int]
        lib.bs_kv_bytes_per_token.argtypes = [C.c_int] + [C.c_int32] * 7
        lib.bs_kv_bytes_per_token.restype = C.c_int64
        lib.bs_builder_split.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.POINTER(SplitInfo)]
        lib.bs_builder_tree_size.argtypes = [C.c_void_p, _i32p, _i32p]
        lib.bs_builder_tree.argtypes = [C.c_void_p] + [_i32p] * 6 + [_i64p, _i64p, _i32p]
        lib.bs_builder_next_batch.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.POINTER(C.POINTER(BatchOwned))]
        lib.bs_builder_emit.argtypes = [C.c_void_p, C.c_int32, _i32p, _i32p, _i32p, C.c_int32, _i32p, _i32p,
                                        C.POINTER(C.POINTER(BatchOwned))]
        lib.bs_sched_create.argtypes = [C.c_void_p, C.POINTER(SchedCfg), _i32p, _i32p, C.POINTER(C.c_void_p)]
        lib.bs_sched_destroy.argtypes = [C.c_void_p]
        lib.bs_sched_destroy.restype = None
        lib.bs_sched_last_error.argtypes = [C.c_void_p]
        lib.bs_sched_last_error.restype = C.c_char_p
        lib.bs_sched_next.argtypes = [C.c_void_p, C.POINTER(C.POINTER(BatchOwned))]
        lib.bs_sched_get_stats.argtypes = [C.c_void_p, C.POINTER(SchedStats)]
        lib.bs_batch_free.argtypes = [C.POINTER(BatchOwned)]
        lib.bs_batch_free.restype = None
        _lib = lib
    return _lib


def check_symbols():
    """Every function the headers declare must be exported by the shared object."""
    lib = raw()
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    if missing:
        raise ImportError("libblendstep.so lacks: " + ", ".join(missing))
    return True


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(_i32p)


def marshal_batch(b):
    """Batch (numpy int32 arrays) -> (BatchDesc, keep-alive list)."""
    arrs = {}
    for name in ("row_start", "kv_len", "page_start", "page_ids", "node_parent", "node_page_start",
                 "node_page_ids", "node_seq_first", "node_seq_count", "seq_leaf_node"):
        a = np.ascontiguousarray(getattr(b, name), dtype=np.int32)
        if a.size == 0:
            a = np.zeros(1, dtype=np.int32)
        arrs[name] = a
    d = BatchDesc(n_seq=b.n_seq, n_prefill=b.n_prefill, n_rows=b.n_rows, n_nodes=b.n_nodes,
                  **{k: _ptr(v) for k, v in arrs.items()})
    return d, arrs


@dataclass
class DeviceState:
    weights: Weights
    keep: list
    x: "object"
    kv_pool: "object"
    n_pages: int


class Layer:
    """One decoder layer's context on one GPU."""

    def __init__(self, shape, device: int = 0, max_positions: int = 0):
        import torch
        self.torch = torch
        self.lib = raw()
        self.shape = shape
        self.device = device
        cfg = LayerCfg(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                       shape.page_size, shape.rms_eps, shape.rope_theta, max_positions)
        h = C.c_void_p()
        rc = self.lib.bs_create(C.byref(cfg), device, C.byref(h))
        if rc != 0:
            raise BlendStepError(rc, (self.lib.bs_last_error(None) or b"").decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.bs_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != 0:
            raise BlendStepError(rc, (self.lib.bs_last_error(self.h) or b"").decode())

    def _stream(self, stream=None):
        s = stream if stream is not None else self.torch.cuda.current_stream(self.device)
        return C.c_void_p(s.cuda_stream)

    # -- device memory ------------------------------------------------------------
    def _bf16(self, a: np.ndarray, transpose: bool = False):
        t = self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:%d" % self.device)
        if transpose:
            t = t.t()
        return t.to(self.torch.bfloat16).contiguous()

    def _bits(self, a: np.ndarray):
        t = self.torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to("cuda:%d" % self.device)
        return t.view(self.torch.bfloat16)

    def upload_weights(self, t) -> tuple:
        w_qkv = self._bf16(t.w_qkv, True)
        w_o = self._bf16(t.w_o, True)
        w_gu = self.torch.cat([self._bf16(t.w_gate, True), self._bf16(t.w_up, True)], dim=0).contiguous()
        w_down = self._bf16(t.w_down, True)
        g1, g2 = self._bf16(t.g_attn), self._bf16(t.g_ffn)
        keep = [w_qkv, w_o, w_gu, w_down, g1, g2]
        w = Weights(*[C.c_void_p(k.data_ptr()) for k in keep])
        return w, keep

    def pack_pool(self, k_bits: np.ndarray, v_bits: np.ndarray):
        n_pages = k_bits.shape[0]
        pool = self.torch.empty(n_pages * self.page_bytes() // 2, dtype=self.torch.bfloat16,
                                device="cuda:%d" % self.device)
        k, v = self._bits(k_bits), self._bits(v_bits)
        self._check(self.lib.bs_kv_pack(self.h, C.c_void_p(k.data_ptr()), C.c_void_p(v.data_ptr()),
                                        C.c_void_p(pool.data_ptr()), n_pages, self._stream()))
        self.torch.cuda.current_stream(self.device).synchronize()
        return pool

    def unpack_pool(self, pool, n_pages: int):
        s = self.shape
        shp = (n_pages, s.page_size, s.n_kv_heads, s.head_dim)
        k = self.torch.empty(shp, dtype=self.torch.bfloat16, device=pool.device)
        v = self.torch.empty(shp, dtype=self.torch.bfloat16, device=pool.device)
        self._check(self.lib.bs_kv_unpack(self.h, C.c_void_p(pool.data_ptr()), C.c_void_p(k.data_ptr()),
                                          C.c_void_p(v.data_ptr()), n_pages, self._stream()))
        self.torch.cuda.current_stream(self.device).synchronize()
        return k, v

    def upload(self, t, batch) -> DeviceState:
        w, keep = self.upload_weights(t)
        x = self._bf16(t.x)
        pool = self.pack_pool(t.k_pool, t.v_pool)
        return DeviceState(w, keep, x, pool, int(t.k_pool.shape[0]))

    def page_bytes(self) -> int:
        return int(self.lib.bs_kv_page_bytes(self.h))

    # -- calls ----------------------------------------------------------------------
    def blend_step(self, dev: DeviceState, batch, flags: int = 0, stream=None, y=None, desc=None):
        d, keep = desc if desc is not None else marshal_batch(batch)
        if y is None:
            y = self.torch.empty_like(dev.x)
        self._check(self.lib.bs_blend_step(self.h, C.byref(dev.weights), C.byref(d), C.c_void_p(dev.x.data_ptr()),
                                           C.c_void_p(y.data_ptr()), C.c_void_p(dev.kv_pool.data_ptr()),
                                           dev.n_pages, self._stream(stream), flags))
        return y

    def blend_layers(self, devs, batch, flags: int = 0, stream=None, y=None, desc=None):
        """The step through len(devs) layers back to back: layer l uses devs[l].weights and
        devs[l].kv_pool; the input is devs[0].x."""
        d, keep = desc if desc is not None else marshal_batch(batch)
        if y is None:
            y = self.torch.empty_like(devs[0].x)
        n = len(devs)
        w = (Weights * n)(*[dv.weights for dv in devs])
        pools = (C.c_void_p * n)(*[dv.kv_pool.data_ptr() for dv in devs])
        self._check(self.lib.bs_blend_layers(self.h, n, w, C.byref(d), C.c_void_p(devs[0].x.data_ptr()),
                                             C.c_void_p(y.data_ptr()), pools, devs[0].n_pages, self._stream(stream), flags))
        return y

    def attention(self, batch, q, kv_pool, n_pages: int, flags: int = 0, stream=None):
        d, keep = marshal_batch(batch)
        out = self.torch.zeros_like(q)
        self._check(self.lib.bs_attention(self.h, C.byref(d), C.c_void_p(q.data_ptr()), C.c_void_p(out.data_ptr()),
                                          C.c_void_p(kv_pool.data_ptr()), n_pages, self._stream(stream), flags))
        return out

    def attention_noalloc(self, batch, q, kv_pool, n_pages: int, out, stream=None):
        """bs_attention_noalloc; `out` is the caller's (nothing is allocated here either)."""
        d, keep = marshal_batch(batch)
        self._check(self.lib.bs_attention_noalloc(self.h, C.byref(d), C.c_void_p(q.data_ptr()), C.c_void_p(out.data_ptr()),
                                                  C.c_void_p(kv_pool.data_ptr()), n_pages, self._stream(stream)))
        return out

    def gemm_nt(self, a, b, stream=None):
        m, k = a.shape
        n = b.shape[0]
        out = self.torch.empty((m, n), dtype=self.torch.bfloat16, device=a.device)
        self._check(self.lib.bs_gemm_nt(self.h, C.c_void_p(a.data_ptr()), C.c_void_p(b.data_ptr()),
                                        C.c_void_p(out.data_ptr()), m, n, k, self._stream(stream)))
        return out

    def validate(self, batch, n_pages: Optional[int] = None) -> int:
        d, keep = marshal_batch(batch)
        return int(self.lib.bs_validate_batch(self.h, C.byref(d), batch.n_pages if n_pages is None else n_pages))

    def last_error(self) -> str:
        return (self.lib.bs_last_error(self.h) or b"").decode()

    def resolve_rows(self, batch):
        d, keep = marshal_batch(batch)
        pg = np.zeros(max(1, batch.n_rows), dtype=np.int32)
        sl = np.zeros(max(1, batch.n_rows), dtype=np.int32)
        self._check(self.lib.bs_resolve_rows(self.h, C.byref(d), _ptr(pg), _ptr(sl)))
        return pg[:batch.n_rows], sl[:batch.n_rows]

    def set_chunk_pages(self, pages: int):
        self._check(self.lib.bs_set_chunk_pages(self.h, pages))

    def get_overlap(self) -> dict:
        k = OverlapKnobs()
        self._check(self.lib.bs_get_overlap(self.h, C.byref(k)))
        return {n: getattr(k, n) for n, _ in OverlapKnobs._fields_}

    def set_overlap(self, **knobs):
        """Change some knobs of the co-scheduled schedule (see bs_overlap_knobs), keeping the others."""
        cur = self.get_overlap()
        for n in knobs:
            if n not in cur:
                raise ValueError("unknown overlap knob " + n)
        cur.update(knobs)
        k = OverlapKnobs(**cur)
        self._check(self.lib.bs_set_overlap(self.h, C.byref(k)))

    def overlap_report(self):
        """KV bytes of the 16-row units per launch of the last co-scheduled step: first attention launch, the
        three carrying GEMM launches, the launch after them."""
        out = (C.c_int64 * 5)()
        self._check(self.lib.bs_overlap_report(self.h, out))
        return [int(v) for v in out]

    def overlap_trace(self, on: bool):
        self._check(self.lib.bs_overlap_trace(self.h, 1 if on else 0))

    def overlap_trace_read(self, launch: int):
        """Records of one launch of the last co-scheduled step: uint64 array [n, 4] (see blendstep.h)."""
        n = C.c_int64()
        self._check(self.lib.bs_overlap_trace_read(self.h, launch, None, 0, C.byref(n)))
        out = np.zeros((max(1, n.value), 4), dtype=np.uint64)
        self._check(self.lib.bs_overlap_trace_read(self.h, launch, out.ctypes.data_as(C.POINTER(C.c_uint64)), n.value,
                                                   C.byref(n)))
        return out[:n.value]

    def set_gemm_tiles(self, variant: int):
        self._check(self.lib.bs_set_gemm_tiles(self.h, variant))

    def profile(self, on: bool):
        self._check(self.lib.bs_profile_enable(self.h, 1 if on else 0))
        self._check(self.lib.bs_profile_reset(self.h))

    def profile_read(self):
        out = {}
        for i, name in enumerate(K_NAMES):
            ms, n = C.c_double(), C.c_int64()
            self._check(self.lib.bs_profile_read(self.h, i, C.byref(ms), C.byref(n)))
            out[name] = (ms.value, n.value)
        return out


class Builder:
    """Host-side batch builder (prefix tree, layer-wise sort, dual scan)."""

    def __init__(self, p_model, kv_bytes, compute, bandwidth, mem_bytes, page_size=16):
        self.lib = raw()
        cm = CostModel(p_model, kv_bytes, compute, bandwidth, mem_bytes, page_size)
        h = C.c_void_p()
        rc = self.lib.bs_builder_create(C.byref(cm), C.byref(h))
        if rc != 0:
            raise BlendStepError(rc, "bs_builder_create failed")
        self.h = h
        self.page_size = page_size

    def close(self):
        if getattr(self, "h", None):
            self.lib.bs_builder_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc < 0:
            raise BlendStepError(rc, (self.lib.bs_builder_last_error(self.h) or b"").decode())
        return rc

    def add(self, tokens, d_est, n_cached=0):
        a = np.ascontiguousarray(tokens, dtype=np.int32)
        return self._check(self.lib.bs_builder_add(self.h, _ptr(a), len(a), int(d_est), int(n_cached)))

    def finalize(self):
        self._check(self.lib.bs_builder_finalize(self.h))

    MEM_MODELS = {"expanded": 0, "shared": 1}

    def set_mem_model(self, name):
        """Memory model behind B ("expanded" or "shared"); before finalize()."""
        if name not in self.MEM_MODELS:
            raise ValueError("unknown memory model " + str(name))
        self._check(self.lib.bs_builder_set_mem_model(self.h, self.MEM_MODELS[name]))

    def split(self, t, budget_tokens=-1):
        """Conditional node splitting; returns what bs_split_info reports."""
        info = SplitInfo()
        self._check(self.lib.bs_builder_split(self.h, int(t), int(budget_tokens), C.byref(info)))
        return dict(n_split=info.n_split, rounds=info.rounds, monotone=bool(info.monotone),
                    recompute_tokens=info.recompute_tokens)

    def tree(self):
        nn, nr = C.c_int32(), C.c_int32()
        self._check(self.lib.bs_builder_tree_size(self.h, C.byref(nn), C.byref(nr)))
        i32 = lambda n: np.zeros(max(1, n), dtype=np.int32)
        i64 = lambda n: np.zeros(max(1, n), dtype=np.int64)
        parent, start, end, req, first, count = (i32(nn.value) for _ in range(6))
        A, B, order = i64(nn.value), i64(nn.value), i32(nr.value)
        p64 = lambda a: a.ctypes.data_as(C.POINTER(C.c_int64))
        self._check(self.lib.bs_builder_tree(self.h, _ptr(parent), _ptr(start), _ptr(end), _ptr(req), _ptr(first),
                                             _ptr(count), p64(A), p64(B), _ptr(order)))
        n = nn.value
        return dict(parent=parent[:n], start=start[:n], end=end[:n], req=req[:n], first_leaf=first[:n],
                    leaf_count=count[:n], A=A[:n], B=B[:n], leaf_order=order[:nr.value])

    def _take(self, out):
        o = out.contents
        b = o.batch
        arr = lambda p, n: np.ctypeslib.as_array(p, shape=(max(1, n),))[:n].copy()
        n_tab = int(b.page_start[b.n_seq]) if b.n_seq else 0
        n_np = int(b.node_page_start[b.n_nodes]) if b.n_nodes else 0
        d = dict(n_seq=b.n_seq, n_prefill=b.n_prefill, n_rows=b.n_rows,
                 row_start=arr(b.row_start, b.n_seq + 1), kv_len=arr(b.kv_len, b.n_seq),
                 page_start=arr(b.page_start, b.n_seq + 1), page_ids=arr(b.page_ids, n_tab),
                 n_nodes=b.n_nodes, node_parent=arr(b.node_parent, b.n_nodes),
                 node_page_start=arr(b.node_page_start, b.n_nodes + 1), node_page_ids=arr(b.node_page_ids, n_np),
                 node_seq_first=arr(b.node_seq_first, b.n_nodes), node_seq_count=arr(b.node_seq_count, b.n_nodes),
                 seq_leaf_node=arr(b.seq_leaf_node, b.n_seq), seq_request=arr(o.seq_request, b.n_seq),
                 n_pages=int(o.n_pages))
        info = {k: getattr(o.info, k) for k, _ in ScanInfo._fields_}
        self.lib.bs_batch_free(out)
        return info, d

    def next_batch(self, prefill_budget=0, decode_budget=0):
        """Returns (info dict, descriptor dict of numpy arrays); the library's copy is freed."""
        out = C.POINTER(BatchOwned)()
        self._check(self.lib.bs_builder_next_batch(self.h, int(prefill_budget), int(decode_budget), C.byref(out)))
        return self._take(out)

    def emit(self, pre, dec):
        """Descriptor of an explicit step: pre = [(request, cached, chunk)], dec = [(request, ctx)]."""
        i32 = lambda v: np.ascontiguousarray(np.asarray(v, dtype=np.int32))
        pr, pc, pk = (i32([x[k] for x in pre]) for k in range(3))
        dr, dc = (i32([x[k] for x in dec]) for k in range(2))
        out = C.POINTER(BatchOwned)()
        self._check(self.lib.bs_builder_emit(self.h, len(pre), _ptr(pr), _ptr(pc), _ptr(pk), len(dec), _ptr(dr), _ptr(dc),
                                             C.byref(out)))
        return self._take(out)[1]


class Scheduler:
    """The multi-step driver over a finalized Builder (bs_sched_*): marshalling only."""

    def __init__(self, builder: Builder, d_true, mem_tokens: int, token_budget: int, n_pages: int, order=None,
                 relocate_pct: int = 200, row_multiple: int = 1):
        self.lib = raw()
        self.builder = builder          # must outlive the scheduler
        cfg = SchedCfg(int(mem_tokens), int(token_budget), int(n_pages), int(relocate_pct), int(row_multiple))
        dt = np.ascontiguousarray(d_true, dtype=np.int32)
        od = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
        h = C.c_void_p()
        rc = self.lib.bs_sched_create(builder.h, C.byref(cfg), _ptr(dt), None if od is None else _ptr(od), C.byref(h))
        if rc != 0:
            raise BlendStepError(rc, "bs_sched_create: invalid arguments")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.bs_sched_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def next_step(self):
        """The next step's descriptor as a dict of numpy arrays, or None when the pool is served."""
        out = C.POINTER(BatchOwned)()
        rc = self.lib.bs_sched_next(self.h, C.byref(out))
        if rc == 1:
            return None
        if rc != 0:
            raise BlendStepError(rc, (self.lib.bs_sched_last_error(self.h) or b"").decode())
        return self.builder._take(out)[1]

    def stats(self) -> dict:
        st = SchedStats()
        rc = self.lib.bs_sched_get_stats(self.h, C.byref(st))
        if rc != 0:
            raise BlendStepError(rc, "bs_sched_get_stats")
        return {n: getattr(st, n) for n, _ in SchedStats._fields_}


class _Api:
    Layer = Layer
    Builder = Builder
    Scheduler = Scheduler
    binding_device_state = DeviceState
    BlendStepError = BlendStepError
    FLAG_SERIAL = FLAG_SERIAL
    FLAG_OVERLAP = FLAG_OVERLAP
    FLAG_PIPELINE = FLAG_PIPELINE
    K_NAMES = K_NAMES
    marshal_batch = staticmethod(marshal_batch)
    raw = staticmethod(raw)


def load():
    raw()
    return _Api


ATTN_VARIANTS = {"mha": 0, "mqa": 1, "gqa": 2, "mla": 3}


def kv_bytes_per_token(variant, n_layers, n_heads=0, head_dim=0, n_kv_heads=0, latent_dim=0, rope_dim=0, elem_bytes=2):
    """bs_kv_bytes_per_token: the cost model's kv_bytes for an attention variant."""
    if variant not in ATTN_VARIANTS:
        raise ValueError("unknown attention variant " + str(variant))
    v = raw().bs_kv_bytes_per_token(ATTN_VARIANTS[variant], n_layers, n_heads, head_dim, n_kv_heads, latent_dim,
                                    rope_dim, elem_bytes)
    if v < 0:
        raise BlendStepError(int(v), "bs_kv_bytes_per_token: invalid arguments")
    return int(v)
