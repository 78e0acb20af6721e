#!/usr/bin/env python3
"""Throughput of one blended decoder-layer step on one MI355X.

A "step" is one call of bs_blend_step: descriptor validation and upload, RMSNorm,
QKV GEMM with RoPE and KV append, prefill and prefix-aware decode attention,
output projection, SwiGLU FFN and both residuals, over one seeded synthetic batch
already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--flags 0|1|3]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16 = 2.5e15  # dense bf16 MFMA, FLOP/s (MI355X datasheet)
PEAK_HBM = 8.0e12        # HBM3E, B/s


def measured_traffic(profile_name, sources):
    """HBM-side bytes per launch of the roofline kernel from the committed counter summary under
    profiles/, or None when the kernel's sources have changed since the counters were taken."""
    import hashlib
    import re
    root = os.path.dirname(os.path.abspath(__file__))
    try:
        text = open(os.path.join(root, "profiles", profile_name)).read()
        h = hashlib.sha256()
        for f in sources:
            h.update(open(os.path.join(root, "paper_2411_16102_amd", "csrc", f), "rb").read())
    except OSError:
        return None
    sha = re.search(r"source_sha256:\s*([0-9a-f]{64})", text)
    val = re.search(r"traffic_bytes_per_launch:\s*(\d+)", text)
    if not sha or not val or sha.group(1) != h.hexdigest():
        return None
    return int(val.group(1))


def overlap_timeline(layer, shape, run_step):
    """One more co-scheduled step with the in-kernel timeline on; per launch: how long the GEMM tiles
    ran, how long the launch lasted, and the KV bytes the attention wavefronts read meanwhile."""
    import numpy as np
    layer.overlap_trace(True)
    run_step()
    names = ["o_proj", "gate_up", "down", "rest_of_queue"]
    per_token = 2 * shape.head_dim * 2   # K and V of one token and KV head
    out = {}
    for k, name in enumerate(names):
        rec = layer.overlap_trace_read(k)
        kind = (rec[:, 2] & np.uint64(0xFF)).astype(int) if len(rec) else np.zeros(0, int)
        used = kind > 0
        if not used.any():
            out[name] = None
            continue
        t0 = int(rec[used, 0].min())
        us = lambda ticks: (int(ticks) - t0) / 100.0    # 100 MHz clock
        tiles, attn = rec[kind == 2], rec[kind == 1]
        info = {"launch_us": us(rec[used, 1].max()), "tiles": int(len(tiles)), "attention_wavefronts": int(len(attn))}
        if len(tiles):
            info["tiles_end_us"] = us(tiles[:, 1].max())
            info["tile_us_mean"] = float(np.mean((tiles[:, 1] - tiles[:, 0]).astype(np.int64))) / 100.0
        if len(attn):
            tokens = (attn[:, 3] >> np.uint64(32)).astype(np.int64)
            units = (attn[:, 3] & np.uint64(0xFFFFFFFF)).astype(np.int64)
            busy = units > 0
            info["kv_bytes"] = int(tokens.sum()) * per_token
            info["units"] = int(units.sum())
            info["attention_end_us"] = us(attn[busy, 1].max()) if busy.any() else 0.0
            info["attention_cus"] = int(len(np.unique((attn[busy, 2] >> np.uint64(8)) & np.uint64(0xFFFFFF0F00)))) if busy.any() else 0
            info["attention_GBps"] = info["kv_bytes"] / max(info["launch_us"], 1e-9) / 1e3
        out[name] = info
    layer.overlap_trace(False)
    return out


def pool_run(args, lib, W, note):
    """The multi-step driver on a synthetic pool (8B-shaped layer): tokens served per second of
    device time under each admission order, over one KV pool that persists across the steps."""
    from paper_2411_16102_amd import engine as E
    shape = W.LLAMA3_8B
    budget = 2560
    reqs = W.synthetic_pool(args.seed, n_groups=args.pool_groups, per_group=12, n_fresh=args.pool_fresh,
                            templates=args.pool_templates)
    prompt = sum(len(r.tokens) for r in reqs)
    outp = sum(r.d_true for r in reqs)
    pages = args.pool_mem_tokens // 16 * 2 + 16384
    stepper = E.GpuStepper(lib, shape, budget, pages, seed=args.seed, flags=max(0, args.flags))
    hw = dict(p_model=8_030_000_000, kv_bytes=shape.kv_bytes_per_token * 32, compute=PEAK_MFMA_BF16, bandwidth=PEAK_HBM)
    for policy in (["blend", "dfs", "random"] if args.pool == "all" else [args.pool]):
        b, sched, split = E.make_scheduler(lib, reqs, hw, args.pool_mem_tokens, budget, pages, policy=policy, seed=args.seed,
                                           split_t=4096 if policy == "blend" else 0, split_budget=int(0.01 * prompt),
                                           mem_model=args.pool_mem_model, row_multiple=args.pool_row_multiple)
        stepper.events = []
        stepper.pool.zero_()
        t0 = time.perf_counter()
        st = E.serve(sched, stepper, progress=lambda s_: note("%s: step %d, %d finished" % (policy, s_["steps"], s_["finished"])))
        ms = stepper.total_ms()
        wall = time.perf_counter() - t0
        print(json.dumps({
            "metric": "pool tokens/s per layer (prompt + output tokens over the device time of all steps)",
            "value": (prompt + outp) / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "policy": policy,
            "schedule": "co-scheduled where a step allows" if stepper.flags else "serial",
            "device_ms": ms, "wall_s": wall, "steps": st["steps"], "requests": len(reqs), "prompt_tokens": prompt,
            "output_tokens": outp, "prefill_rows": st["prefill_rows"], "prompt_tokens_skipped": st["prompt_tokens_skipped"],
            "decode_rows": st["decode_rows"], "mean_rows_per_step": st["rows"] / max(1, st["steps"]),
            "peak_kv_tokens": st["peak_tokens"], "peak_pages": st["peak_pages"], "kv_capacity_tokens": args.pool_mem_tokens,
            "mem_left": st["mem_left"], "mem_right": st["mem_right"],
            "split": split, "mem_model": args.pool_mem_model, "row_multiple": args.pool_row_multiple, "templates": args.pool_templates,
            "relocated": st["relocated"], "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "pool(seed=%d, groups=%d, fresh=%d)" % (args.seed, args.pool_groups, args.pool_fresh), "token_budget": budget,
                       "d_model": shape.d_model, "d_ffn": shape.d_ffn}}), flush=True)


def cpu_baseline(shape, batch, tens, target_flops=1.2e12):
    """The oracle, as it stands, on a bounded sample of the same batch: whole
    prefill segments and evenly spaced decode sequences in the batch's own
    prefill:decode proportion."""
    import numpy as np
    from oracle import layer as oracle_layer
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    q_len = batch.q_len()
    n_pre_rows = int(batch.row_start[batch.n_prefill])
    target_rows = target_flops / (2.0 * shape.matrix_params)   # about 10-20 s of float64 BLAS on 16 cores
    frac = min(1.0, target_rows / max(1, batch.n_rows))
    rows = []
    pre_target = frac * n_pre_rows
    took = 0
    for s in range(batch.n_prefill):
        if took >= pre_target:
            break
        rows.extend(range(int(batch.row_start[s]), int(batch.row_start[s + 1])))
        took += int(q_len[s])
    n_dec = batch.n_seq - batch.n_prefill
    dec_take = int(round(frac * n_dec)) if n_dec else 0
    if n_dec and dec_take == 0:
        dec_take = 1
    if dec_take:
        pick = np.unique(np.linspace(0, n_dec - 1, dec_take).astype(int))
        rows.extend(int(batch.row_start[batch.n_prefill + i]) for i in pick)
    t0 = time.perf_counter()
    oracle_layer.layer_step(shape, tens, batch, rows=rows)
    dt = time.perf_counter() - t0
    return {"value": len(rows) / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d of %d rows (%d prefill rows in whole segments + %d decode sequences), %.1f s, float64 numpy"
                      % (len(rows), batch.n_rows, took, len(rows) - took, dt)}, rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="blended_8b")
    ap.add_argument("--flags", type=int, default=-1, help="0 serial, 1 overlap, 3 overlap with the layers of a --layers call pipelined, -1 pick the faster of 0 and 1 in warm-up")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk-pages", type=int, default=0)
    ap.add_argument("--overlap-knobs", default="",
                    help="knobs of the co-scheduled schedule as name=value,name=value (see bs_overlap_knobs)")
    ap.add_argument("--gemm-tiles", type=int, default=0, help="force one GEMM tile shape (0: cost model)")
    ap.add_argument("--layers", type=int, default=1,
                    help="a step = this many layers back to back through bs_blend_layers (same weights and pool "
                         "for every layer: timing only); value stays per layer")
    ap.add_argument("--pool", default="",
                    help="instead of one workload: serve a synthetic request pool to completion with the multi-step "
                         "driver, admission order blend | dfs | random | all (one JSON line each)")
    ap.add_argument("--pool-mem-tokens", type=int, default=200_000, help="KV capacity of the pool run, in tokens")
    ap.add_argument("--pool-groups", type=int, default=24, help="prefix groups of 12 requests (short, medium, long outputs in turn)")
    ap.add_argument("--pool-row-multiple", type=int, default=1,
                    help="steps of more rows than this are cut to a multiple of it (1: off)")
    ap.add_argument("--pool-mem-model", default="expanded", choices=["expanded", "shared"],
                    help="memory model of the densities: the paper's, or shared prefix pages charged once per step")
    ap.add_argument("--pool-fresh", type=int, default=1500, help="prompt-heavy requests without shared prefix")
    ap.add_argument("--pool-templates", default="by_kind", choices=["by_kind", "shuffled"],
                    help="numbering of the datasets' template tokens: the order that hurts the prefix-DFS baseline, or a random one")
    ap.add_argument("--overlap-trace", action="store_true",
                    help="with the co-scheduled schedule: add the in-kernel timeline of one more step to the line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB elementwise copy (for scaling HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards by independent replicas, one "
              "process and one request pool per GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2411_16102_amd as pkg
    from paper_2411_16102_amd import workloads as W

    def note(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    lib = pkg.load()
    if args.pool:
        return pool_run(args, lib, W, note)
    note("generating inputs for " + args.workload)
    shape, make_batch = W.CONFIGS[args.workload]
    batch = make_batch(seed=args.seed)
    work = W.work_of(shape, batch)
    tens = W.make_tensors(shape, batch, args.seed)
    layer = lib.Layer(shape, device=0)
    if args.chunk_pages:
        layer.set_chunk_pages(args.chunk_pages)
    if args.gemm_tiles:
        layer.set_gemm_tiles(args.gemm_tiles)
    if args.overlap_knobs:
        layer.set_overlap(**{kv.split("=")[0]: int(kv.split("=")[1]) for kv in args.overlap_knobs.split(",")})
    note("uploading")
    dev = layer.upload(tens, batch)
    desc = lib.marshal_batch(batch)
    if args.copy_calibration:
        # a plain copy of known size: reads 2^30 bytes and writes 2^30 bytes per launch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    note("timing")
    y = torch.empty_like(dev.x)

    def run_once(flags):
        if args.layers > 1:
            layer.blend_layers([dev] * args.layers, batch, flags=flags, y=y, desc=desc)
        else:
            layer.blend_step(dev, batch, flags=flags, y=y, desc=desc)

    def run(n, flags):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            run_once(flags)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / max(1, n)

    flags = args.flags
    schedules_ms = None
    if flags < 0:
        # both schedules, alternating, the same number of steps each; the faster one is timed
        n_try = max(5, args.warmup)
        run(max(2, args.warmup // 2), 0)
        run(max(2, args.warmup // 2), 1)
        t_serial = min(run(n_try, 0), run(n_try, 0))
        t_overlap = min(run(n_try, 1), run(n_try, 1))
        flags = 1 if t_overlap < t_serial else 0
        schedules_ms = {"serial": t_serial * 1e3 / args.layers, "co_scheduled": t_overlap * 1e3 / args.layers}
    run(args.warmup, flags)
    sec = run(args.steps, flags) / args.layers

    # spread of single calls: the same loop once more with a pair of events around every call
    stream = torch.cuda.current_stream()
    pairs = []
    for _ in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        run_once(flags)
        e1.record(stream)
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    per_call = np.sort(np.array([a.elapsed_time(b) for a, b in pairs])) / args.layers
    spread = {"p10": float(np.percentile(per_call, 10)), "p50": float(np.percentile(per_call, 50)),
              "p90": float(np.percentile(per_call, 90))}

    # per-kernel durations: the same loop again with HIP events around every kernel class
    layer.profile(True)
    run(args.steps, flags)
    prof = layer.profile_read()
    layer.profile(False)
    carried = layer.overlap_report() if flags else None   # of the last step of that pass
    if schedules_ms is not None:
        # how much any overlap could give at most: the serial step without its attention launches
        n0 = max(5, args.warmup)
        layer.profile(True)
        run(n0, 0)
        p0 = layer.profile_read()
        layer.profile(False)
        attn_ms = sum(p0[k][0] for k in ("attn_prefill", "attn_decode", "attn_merge")) / (n0 * args.layers)
        schedules_ms["serial_attention_launches"] = attn_ms
        schedules_ms["serial_if_attention_were_free"] = schedules_ms["serial"] - attn_ms
    # per kernel class: milliseconds per step and layer (all launches of the class added up)
    kernels = {k: {"ms": ms / (args.steps * args.layers), "launches_per_step": n / (args.steps * args.layers)}
               for k, (ms, n) in prof.items()}

    T, d, f = batch.n_rows, shape.d_model, shape.d_ffn
    Tp = int(batch.row_start[batch.n_prefill])
    hd = shape.n_q_heads * shape.head_dim
    t_flop = work["flops"] / PEAK_MFMA_BF16
    t_byte = work["bytes_once"] / PEAK_HBM
    bound = "mfma" if t_flop >= t_byte else "hbm"
    co = bool(flags) and kernels["gemm_decode_rows"]["launches_per_step"] > 0   # the step took the co-scheduled path
    rows_g = Tp if co else T     # rows of the output-projection and gate/up launches (co-scheduled: the prefill rows)
    rows_dn = Tp if (co and layer.get_overlap()["carry_down"]) else T
    kv_bytes = work["kv_tokens_once"] * shape.kv_bytes_per_token

    def mfma(name, cls, flops, traffic_file=None, extra=None, operand_bytes=0.0):
        ms = kernels[cls]["ms"]
        if ms <= 0:
            return None
        r = {"bound": "mfma", "kernel": name, "ms": ms, "achieved": flops / (ms * 1e-3) / 1e12, "peak": PEAK_MFMA_BF16 / 1e12,
             "unit": "TFLOP/s", "traffic": (measured_traffic(traffic_file, ["gemm.hip", "gemm.hpp", "common.hpp", "attn_device.hpp"])
                                            if traffic_file else None)}
        r["frac"] = r["achieved"] / r["peak"]
        if extra:
            # A launch that carries decode attention does two kinds of algorithmic work at once: the GEMM's
            # flops on the tile CUs and the KV bytes (plus the GEMM's own operands, each once) on the memory
            # system.  Its roofline time is the larger of the two, and that side names the bound.
            r.update(extra)
            nbytes = extra["carried_kv_bytes"] + operand_bytes
            r["mfma_frac"] = r["frac"]
            r["hbm_frac"] = nbytes / (ms * 1e-3) / PEAK_HBM
            r["algorithmic_flops"], r["algorithmic_bytes"] = flops, nbytes
            if r["hbm_frac"] > r["mfma_frac"]:
                r.update({"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                          "frac": r["hbm_frac"]})
        return r

    def hbm(name, cls, nbytes, traffic_file=None):
        ms = kernels[cls]["ms"]
        if ms <= 0:
            return None
        r = {"bound": "hbm", "kernel": name, "ms": ms, "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
             "traffic": (measured_traffic(traffic_file, ["attn.hip", "attn.hpp", "attn_device.hpp", "common.hpp"]) if traffic_file else None)}
        r["frac"] = r["achieved"] / r["peak"]
        return r

    def riding(k):   # KV bytes per second that the attention workgroups of carrying launch k read beside its tiles
        cls = ["gemm_o", "gemm_gate_up", "gemm_down"][k]
        return {"carried_kv_bytes": carried[1 + k], "carried_kv_GBps": carried[1 + k] / (kernels[cls]["ms"] * 1e-3) / 1e9}

    tag = " of the prefill rows, carrying decode attention" if co else ""
    per_kernel = [
        mfma("gemm_qkv (RMSNorm factor, RoPE, KV append)", "gemm_qkv", 2.0 * T * d * shape.n_qkv),
        # (operand bytes of a carrying launch: activations in, weights, result out, each once; x1 leaves the
        # output projection in fp32 and as bf16(x1 * gain), and the down projection reads it back in fp32)
        mfma("gemm_o (residual, norm statistics)" + tag, "gemm_o", 2.0 * rows_g * hd * d, None, riding(0) if co else None,
             2.0 * rows_g * hd + 2.0 * hd * d + rows_g * d * (2.0 + 4.0 + 2.0)),
        mfma("gemm_gate_up (SwiGLU epilogue)" + tag, "gemm_gate_up", 2.0 * rows_g * d * 2 * f,
             ("blended_8b_coscheduled_gate_up_hbm_traffic.txt" if co else "blended_8b_gemm_gate_up_hbm_traffic.txt")
             if args.workload == "blended_8b" else None,
             riding(1) if co else None, 2.0 * rows_g * d + 2.0 * d * 2 * f + 2.0 * rows_g * f),
        mfma("gemm_down (residual)" + (tag if rows_dn != T else ""), "gemm_down", 2.0 * rows_dn * f * d, None,
             riding(2) if (co and rows_dn != T) else None, 2.0 * rows_dn * f + 2.0 * f * d + rows_dn * d * (4.0 + 2.0)),
        mfma("output projection, gate/up and down of the decode rows", "gemm_decode_rows",
             2.0 * (T - Tp) * (hd * d + 2 * d * f) + 2.0 * (T - rows_dn) * f * d) if co else None,
    ]
    if co:
        per_kernel.append(hbm("attention of the prefill rows, the wide decode items and the decode units that do not ride",
                              "attn_decode", kv_bytes - sum(carried[1:])))
    elif kernels["attn_decode"]["ms"] > 0:
        per_kernel.append(hbm("attention (paged, prefix-aware; prefill rows in the same launch)" if kernels["attn_prefill"]["ms"] == 0
                              else "decode_attn (paged, prefix-aware)", "attn_decode",
                              kv_bytes if kernels["attn_prefill"]["ms"] == 0 else
                              kv_bytes - float(np.sum(batch.kv_len[:batch.n_prefill])) * shape.kv_bytes_per_token,
                              {"blended_8b": "blended_8b_attention_hbm_traffic.txt",
                               "decode_8b": "decode_8b_decode_attn_trace_and_hbm_traffic.txt"}.get(args.workload)))
    per_kernel = [r for r in per_kernel if r]
    # the dominant kernel = the longest launch of the step; the bound-side kernel = the longest one of the
    # kind that bounds the whole step (a GEMM where the step is MFMA-bound, attention where it is HBM-bound)
    roofline = max(per_kernel, key=lambda r: r["ms"])
    def as_mfma(r):   # a carrying launch seen from its GEMM side
        if r["bound"] == "mfma" or "mfma_frac" not in r:
            return r
        return dict(r, bound="mfma", achieved=r["algorithmic_flops"] / (r["ms"] * 1e-3) / 1e12, peak=PEAK_MFMA_BF16 / 1e12,
                    unit="TFLOP/s", frac=r["mfma_frac"])
    side = [as_mfma(r) if bound == "mfma" else r for r in per_kernel]
    side = [r for r in side if r["bound"] == bound]
    roofline_bound_side = max(side, key=lambda r: r["ms"]) if side else None

    out = {
        "metric": "blended-step tokens/s per layer", "value": T / sec, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
        "ms_per_call_by_events": spread,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "rows": T, "prefill_rows": int(batch.row_start[batch.n_prefill]),
                   "decode_seqs": batch.n_seq - batch.n_prefill, "prefix_nodes": batch.n_nodes,
                   "layers_per_call": args.layers, "d_model": d, "n_q_heads": shape.n_q_heads, "n_kv_heads": shape.n_kv_heads,
                   "head_dim": shape.head_dim, "d_ffn": f, "seed": args.seed,
                   "schedule": ("co-scheduled" if co else "serial")},
        "step_roofline": {"flops": work["flops"], "bytes": work["bytes_once"], "bytes_if_expanded": work["bytes_expanded"],
                          "t_flop_us": t_flop * 1e6, "t_byte_us": t_byte * 1e6, "bound": bound,
                          "frac": max(t_flop, t_byte) / sec},
        "roofline": roofline,
        "roofline_bound_side": roofline_bound_side,
        "roofline_per_kernel": [{k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()} for r in per_kernel],
        "kernels_ms": {k: round(v["ms"], 4) for k, v in kernels.items()},
    }
    if schedules_ms:
        # the step's compute-bound and memory-bound kernels one after the other (serial) against co-scheduled
        out["schedules_ms"] = {k: round(v, 4) for k, v in schedules_ms.items()}
        out["step_roofline"]["frac_if_attention_were_free"] = max(t_flop, t_byte) / (schedules_ms["serial_if_attention_were_free"] * 1e-3)
    if flags:
        out["overlap_kv_bytes"] = carried
        if args.overlap_trace:
            out["overlap_timeline"] = overlap_timeline(layer, shape, lambda: run_once(flags))
    if batch.n_prefill and batch.n_seq > batch.n_prefill and kernels["attn_prefill"]["launches_per_step"] == 0:
        out["kernels_note"] = "attn_decode is the one launch that runs prefill and decode attention together"
    if not args.no_cpu_baseline:
        note("timing the CPU oracle on a sample")
        out["cpu_baseline"], _ = cpu_baseline(shape, batch, tens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
