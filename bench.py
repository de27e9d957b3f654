"""Benchmark of the EliteKV decode hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
  elitekv_append of the batch's new tokens (down-projection + selective RoPE, written into the
  cache planes) followed by elitekv_decode_attn over the whole cached context.
The default workload is the 7B shape at 25 % cache, batch 1, 32K context.  Inputs are resident
in HBM before the timed region.  The timed steps cycle over several distinct copies of the
cache planes (>= 1 GiB in total) and of the weights (>= 512 MB in total: a model's next layer brings its
own) so that the 256 MB Infinity Cache cannot serve the reads.

Order of a run: the oracle's timing on the host and the companion measurements (streaming ceiling,
uncompressed attention, several queries, whole block, prefill-sized calls, search) first, then the
headline region: W untimed warm-up steps, a synchronisation, exactly K timed steps, a synchronisation.

Prints one JSON line.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_VALU_PEAK_TFLOPS = 157.3       # 256 compute units x 4 SIMDs x 64 lanes x 2 flops at 2.4 GHz
METRIC = "decode attn HBM GB/s (% of peak) + tokens/s, 7B shape 25% cache, 32K ctx"


def counted_traffic(workload):
    """HBM bytes per launch of the dominant kernel as counted by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each
    scaled by what the same counter reads for a plain copy of known size): read from the committed summary of
    that workload, profiles/attn_mfma_<workload>.md, which carries one line
        traffic_bytes_per_launch: <integer>
    Returns (bytes or None, "file name @ first 12 hex digits of its sha1" or None): no summary, no number."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", "attn_mfma_%s.md" % workload)
    try:
        text = open(path, "rb").read()
    except OSError:
        return None, None
    m = re.search(rb"^traffic_bytes_per_launch:\s*(\d+)\s*$", text, re.M)
    if not m:
        return None, None
    return int(m.group(1)), "profiles/%s @ %s" % (os.path.basename(path), hashlib.sha1(text).hexdigest()[:12])


class HipEvents:
    """HIP events through the runtime's C API, recorded on the stream the kernels run on."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self):
        ev = C.c_void_p()
        rc = self.hip.hipEventCreate(C.byref(ev))
        assert rc == 0, "hipEventCreate failed: %d" % rc
        return ev

    def record(self, ev, stream):
        rc = self.hip.hipEventRecord(ev, C.c_void_p(stream))
        assert rc == 0, "hipEventRecord failed: %d" % rc

    def elapsed_ms(self, a, b):
        self.hip.hipEventSynchronize(b)
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), a, b)
        assert rc == 0, "hipEventElapsedTime failed: %d" % rc
        return float(ms.value)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="7b_25_b1_s32768")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-comparators", action="store_true",
                    help="only the decode step: skip the comparators and the multiquery / search / prefill fields")
    ap.add_argument("--prefill-tokens", type=int, default=2048,
                    help="tokens of the append_prefill field (the matrix-core append)")
    ap.add_argument("--no-multiquery", action="store_true",
                    help="skip the multiquery field (it launches the attention kernel in another configuration)")
    ap.add_argument("--splits", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (nothing in it is distributed); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import elitekv_synth as synth
    import paper_2503_01586_amd as ekv

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.CONFIGS[args.workload]
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    esz = 2 if cfg.dtype == "bf16" else 4
    B, S, n_h, d_h, r, d_c, d = cfg.batch, cfg.context, cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c, cfg.d_model
    dims = ekv.make_dims(d, n_h, d_h, r, d_c, cfg.dtype, cfg.rope_base)
    row_bytes = (2 * r * n_h + d_c) * esz
    cache_bytes = B * S * row_bytes                                   # both planes, read once per call
    n_copies = max(2, -(-(1 << 30) // cache_bytes))

    rng = synth.rng_for(cfg.index)
    idx_h = synth.draw_elite_idx(rng, n_h, d_h, r)
    assert ekv.elitekv_validate_elite_idx(dims, idx_h) == 0
    d_ck = cfg.d_ck                                   # > 0: separated latents, a cache row is [c^k | c^v]
    if d_ck:
        W_ke, W_dkv, W_uk, _ = synth.draw_weights(rng, d, n_h, d_h, r, d_ck)          # A^k, B^k_S
        _, W_dkv2, _, W_uv = synth.draw_weights(rng, d, n_h, d_h, r, d_c - d_ck)      # A^v, B^v_S
        W_dkv2_d = torch.from_numpy(np.ascontiguousarray(W_dkv2)).to(dt).to(dev)
    else:
        W_ke, W_dkv, W_uk, W_uv = synth.draw_weights(rng, d, n_h, d_h, r, d_c)
        W_dkv2_d = None
    q_h = synth.draw_query(rng, B, n_h, d_h)
    x_h = synth.draw_hidden(rng, B, d)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(dev)
    W_ke_d, W_dkv_d, W_uk_d, W_uv_d, q_d, x_d = map(to_dev, (W_ke, W_dkv, W_uk, W_uv, q_h, x_h))
    idx_d = torch.from_numpy(idx_h).to(dev)
    # Weight copies the timed steps rotate over, like the plane copies: a model's next layer brings its own
    # weights, so a step must not find them in the 256 MB Infinity Cache from the step before.
    w_bytes = sum(t.numel() * t.element_size() for t in (W_ke_d, W_dkv_d, W_uk_d, W_uv_d) + ((W_dkv2_d,) if d_ck else ()))
    n_wcopies = max(2, -(-(512 << 20) // w_bytes))
    wsets = [(W_ke_d, W_dkv_d, W_dkv2_d, W_uk_d, W_uv_d)]
    for _ in range(n_wcopies - 1):
        wsets.append(tuple(None if t is None else t.clone() for t in wsets[0]))
    rows = B * S
    planes = []
    host_planes0 = None
    for i in range(n_copies):
        prng = synth.rng_for(cfg.index, stream=100 + i)
        ke_h = prng.standard_normal((rows, n_h, 2 * r), dtype=np.float32)
        c_h = prng.standard_normal((rows, d_c), dtype=np.float32)
        ke_t, c_t = torch.from_numpy(ke_h).to(dt), torch.from_numpy(c_h).to(dt)
        if i == 0:
            host_planes0 = (ke_t, c_t)
        planes.append((ke_t.to(dev), c_t.to(dev)))
    pos_d = torch.full((B,), S - 1, dtype=torch.int32, device=dev)
    slot_d = (torch.arange(B, dtype=torch.int64, device=dev) * S + (S - 1))
    seq_d = torch.full((B,), S, dtype=torch.int32, device=dev)
    out_d = torch.empty(B, n_h, d_h, dtype=dt, device=dev)
    if d_ck:
        nws, naws = (ekv.elitekv_slrd_decode_workspace_bytes(dims, d_ck, B, S, args.splits),
                     ekv.elitekv_slrd_append_workspace_bytes(dims, d_ck, B))
    else:
        nws, naws = ekv.elitekv_decode_workspace_bytes(dims, B, S, args.splits), ekv.elitekv_append_workspace_bytes(dims, B)
    nsws = (ekv.elitekv_slrd_decode_step_workspace_bytes(dims, d_ck, B, S, args.splits) if d_ck
            else ekv.elitekv_decode_step_workspace_bytes(dims, B, S, args.splits))
    ws_d = torch.empty(max(nws, nsws, 16), dtype=torch.uint8, device=dev)   # the step's workspace starts with the decode's
    aws_d = torch.empty(max(naws, 16), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    ev = HipEvents()

    def step(i, same_weights=False):
        ke_p, c_p = planes[i % n_copies]
        Wke, Wdkv, Wdkv2, Wuk, Wuv = wsets[0 if same_weights else i % n_wcopies]
        if d_ck:
            ekv.elitekv_slrd_decode_step(dims, d_ck, x_d, q_d, pos_d, slot_d, seq_d, S, S, Wke, Wdkv, Wdkv2,
                                         Wuk, Wuv, idx_d, ke_p, c_p, out_d, ws_d, n_splits=args.splits,
                                         stream=stream)
        else:
            ekv.elitekv_decode_step(dims, x_d, q_d, pos_d, slot_d, seq_d, S, S, Wke, Wdkv, Wuk, Wuv, idx_d,
                                    ke_p, c_p, out_d, ws_d, n_splits=args.splits, stream=stream)

    def step_two_calls(i):
        ke_p, c_p = planes[i % n_copies]
        Wke, Wdkv, Wdkv2, Wuk, Wuv = wsets[i % n_wcopies]
        if d_ck:
            ekv.elitekv_slrd_append(dims, d_ck, x_d, pos_d, slot_d, Wke, Wdkv, Wdkv2, idx_d, ke_p, c_p,
                                    ws=aws_d, stream=stream)
            ekv.elitekv_slrd_decode_attn(dims, d_ck, q_d, pos_d, seq_d, S, S, Wuk, Wuv, idx_d, ke_p, c_p, out_d,
                                         ws_d, n_splits=args.splits, stream=stream)
        else:
            ekv.elitekv_append(dims, x_d, pos_d, slot_d, Wke, Wdkv, idx_d, ke_p, c_p, ws=aws_d, stream=stream)
            ekv.elitekv_decode_attn(dims, q_d, pos_d, seq_d, S, S, Wuk, Wuv, idx_d, ke_p, c_p, out_d, ws_d,
                                    n_splits=args.splits, stream=stream)

    # The companion measurements (streaming ceiling, uncompressed attention, several queries, the whole block, the
    # prefill-sized calls, the search) and the oracle on the host run FIRST, the headline step LAST: the chip needs some
    # 15 ms of sustained kernels after an idle period before its kernels run at their steady speed (a kernel trace shows
    # every kernel of the step 4-5 % slower until then), and a short run (the driver's: 5 + 20 steps, about a
    # millisecond) that follows the host-side set-up directly would be timed entirely in that start-up phase.
    extras = {}
    cpu_res = None
    if not args.no_cpu_baseline:
        cpu_res = cpu_baseline(cfg, idx_h, W_ke_d, W_dkv_d, W_dkv2_d, W_uk_d, W_uv_d, q_d, x_d, host_planes0, cache_bytes)
    if not args.no_comparators:
        if not d_ck and B < 8:
            extras["block_step"] = block_step(ekv, ev, cfg, dims, planes, x_d, pos_d, slot_d, seq_d, W_ke_d, W_dkv_d, W_uk_d,
                                              W_uv_d, idx_d, dev, dt, stream, cache_bytes, args)
        extras["prefill_attn"] = prefill_attn(ekv, ev, cfg, dims, planes, W_uk_d, W_uv_d, idx_d, dev, dt, stream,
                                              T=args.prefill_tokens)
        extras["ropelite_search"] = ropelite_search(ekv, ev, cfg, dev, stream)
        extras["ropelite_search"]["at_2048_tokens"] = ropelite_search(ekv, ev, cfg, dev, stream, T=2048, iters=2)
        extras["append_prefill"] = append_prefill(ekv, ev, cfg, dims, W_ke_d, W_dkv_d, W_dkv2_d, idx_d, dev, dt, stream,
                                                  T=args.prefill_tokens)
        extras["comparators"] = comparators(ekv, ev, cfg, dims, planes, q_d, pos_d, seq_d, dev, dt, stream,
                                            cache_bytes, args)
        if not d_ck and not args.no_multiquery:
            extras["multiquery"] = multiquery(ekv, ev, cfg, dims, planes, W_uk_d, W_uv_d, idx_d, dev, dt, stream,
                                              cache_bytes)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = ev.create(), ev.create()
    ev.record(e0, stream)
    for i in range(args.steps):
        step(i)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms_per_step = ev.elapsed_ms(e0, e1) / args.steps
    # four more regions of the same K steps: spread of the measurement (value comes from the first)
    reps = [ms_per_step]
    for _ in range(4):
        ev.record(e0, stream)
        for i in range(args.steps):
            step(i)
        ev.record(e1, stream)
        torch.cuda.synchronize()
        reps.append(ev.elapsed_ms(e0, e1) / args.steps)
    reps.sort()
    # the same K steps with ONE set of weights (they then stay in the Infinity Cache from step to step)
    ev.record(e0, stream)
    for i in range(args.steps):
        step(i, same_weights=True)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms_same_weights = ev.elapsed_ms(e0, e1) / args.steps
    # the same work through the two separate entry points (append, then attention), for reference
    for i in range(args.warmup):
        step_two_calls(i)
    torch.cuda.synchronize()
    ev.record(e0, stream)
    for i in range(args.steps):
        step_two_calls(i)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms_two_calls = ev.elapsed_ms(e0, e1) / args.steps
    # elitekv_decode_attn alone (query preparation, split attention, merge + up-projection), the call the
    # north star prices, over the same rotating plane and weight copies
    def attn_call(i):
        ke_p, c_p = planes[i % n_copies]
        _, _, _, Wuk, Wuv = wsets[i % n_wcopies]
        if d_ck:
            ekv.elitekv_slrd_decode_attn(dims, d_ck, q_d, pos_d, seq_d, S, S, Wuk, Wuv, idx_d, ke_p, c_p, out_d, ws_d,
                                         n_splits=args.splits, stream=stream)
        else:
            ekv.elitekv_decode_attn(dims, q_d, pos_d, seq_d, S, S, Wuk, Wuv, idx_d, ke_p, c_p, out_d, ws_d,
                                    n_splits=args.splits, stream=stream)
    for i in range(args.warmup):
        attn_call(i)
    torch.cuda.synchronize()
    ev.record(e0, stream)
    for i in range(args.steps):
        attn_call(i)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms_attn_call = ev.elapsed_ms(e0, e1) / args.steps

    # dominant kernel (the split attention kernel): K launches of that stage alone, back to back on
    # the stream over the same rotating plane copies, between ONE pair of HIP events (an event pair
    # around every single launch adds several microseconds of marker time to a 30 us kernel).  The
    # workspace holds the prepared query of the full calls above; it does not depend on the planes.
    def attn_only(i):
        ke_p, c_p = planes[i % n_copies]
        ekv.elitekv_decode_attn_stages(dims, q_d, pos_d, seq_d, S, S, W_uk_d, W_uv_d, idx_d, ke_p, c_p, out_d, ws_d,
                                       2, n_splits=args.splits, stream=stream, d_ck=d_ck)
    step_two_calls(0)          # a full elitekv_decode_attn with these arguments leaves the prepared query behind
    for i in range(args.warmup):
        attn_only(i)
    torch.cuda.synchronize()
    # At least 500 launches per event pair (14 ms), with a few untimed ones queued ahead of the first event: a
    # region that opens on an idle queue pays some 30 us before its launches follow each other back to back,
    # which is 1 % of 100 launches of 27 us and 5 % of 20.
    n_k = max(args.steps, 500)
    k_runs = []
    for rep in range(5):
        for i in range(3):
            attn_only(i)
        ev.record(e0, stream)
        for i in range(n_k):
            attn_only(3 + i)
        ev.record(e1, stream)
        torch.cuda.synchronize()
        k_runs.append(ev.elapsed_ms(e0, e1) / n_k)
    k_runs.sort()
    k_avg_ms = sum(k_runs) / len(k_runs)
    # restore the output of a full step for the finiteness check below
    step(0)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out_d.float()).all()), "non-finite output"

    value_gbs = cache_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = cache_bytes / (k_avg_ms * 1e-3) / 1e9
    traffic, traffic_src = counted_traffic(cfg.name)
    result = {
        "metric": METRIC, "value": round(value_gbs, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "batch": B, "context": S, "d_model": d, "n_heads": n_h, "head_dim": d_h,
                   "r": r, "d_c": d_c, "cache_fraction": (2 * r * n_h + d_c) / (2 * n_h * d_h),
                   "variant": "S-LRD (d_ck %d, d_cv %d)" % (d_ck, d_c - d_ck) if d_ck else "J-LRD",
                   "step": ("elitekv_slrd_decode_step (= elitekv_slrd_append(T=batch) + elitekv_slrd_decode_attn)" if d_ck
                            else "elitekv_decode_step (= elitekv_append(T=batch) + elitekv_decode_attn)"),
                   "plane_copies": n_copies, "weight_copies": n_wcopies,
                   "n_splits": ekv.elitekv_decode_auto_splits(dims, B, S) if args.splits == 0 else args.splits},
        "pct_of_hbm_peak": round(100.0 * value_gbs / HBM_PEAK_GBS, 2),
        "tokens_per_s": round(B / (ms_per_step * 1e-3), 1),
        "ms_per_step_median": round(reps[len(reps) // 2], 5), "ms_per_step_min": round(reps[0], 5),
        "ms_per_step_two_calls": round(ms_two_calls, 5),
        "ms_decode_attn_call": round(ms_attn_call, 5),
        "decode_attn_call_GBs": round(cache_bytes / (ms_attn_call * 1e-3) / 1e9, 2),
        "ms_per_step_one_weight_set": round(ms_same_weights, 5),
        "roofline": {"bound": "hbm", "kernel": "split attention kernel of elitekv_decode_attn",
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": cache_bytes, "avg_launch_ms": round(k_avg_ms, 5),
                     "median_launch_ms": round(k_runs[len(k_runs) // 2], 5), "min_launch_ms": round(k_runs[0], 5),
                     "launches_timed": 5 * n_k},
    }

    if not args.no_comparators:
        result.update(extras)
        # the step against the roofline with everything it has to read once (cache + the four weight
        # matrices), and against the measured streaming ceiling of this machine
        other = 2 * (d * (2 * r * n_h + d_c) + (d_ck or d_c) * n_h * (d_h - 2 * r) + (d_c - d_ck) * n_h * d_h)
        ceil_gbs = result["comparators"]["stream_read_GBs"]
        result["fractions"] = {
            "step_cache_bytes_of_peak": round(value_gbs / HBM_PEAK_GBS, 4),
            "step_all_algorithmic_bytes_of_peak": round((cache_bytes + other) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "step_cache_bytes_of_stream_ceiling": round(value_gbs / ceil_gbs, 4),
            "attention_kernel_of_peak": round(achieved / HBM_PEAK_GBS, 4),
            "attention_kernel_of_stream_ceiling": round(achieved / ceil_gbs, 4),
            "weight_bytes_per_step": other, "stream_ceiling_GBs": ceil_gbs}
    if cpu_res is not None:
        result["cpu_baseline"] = cpu_res
    print(json.dumps(result))


def comparators(ekv, ev, cfg, dims, planes, q_d, pos_d, seq_d, dev, dt, stream, cache_bytes, args):
    """Streaming-read ceiling over the same planes, and ordinary RoPE-MHA decode at the same shape."""
    import torch
    B, S, n_h, d_h = cfg.batch, cfg.context, cfg.n_heads, cfg.head_dim
    out = {}
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    n = max(20, args.steps // 4)
    for i in range(5):
        ekv.elitekv_stream_read(planes[i % len(planes)][1], sink, stream=stream)
    e0, e1 = ev.create(), ev.create()
    ev.record(e0, stream)
    nbytes = 0
    for i in range(n):
        ke_p, c_p = planes[i % len(planes)]
        ekv.elitekv_stream_read(c_p, sink, stream=stream)
        ekv.elitekv_stream_read(ke_p, sink, stream=stream)
        nbytes += c_p.numel() * c_p.element_size() + ke_p.numel() * ke_p.element_size()
    ev.record(e1, stream)
    torch.cuda.synchronize()
    out["stream_read_planes_GBs"] = round(nbytes / (ev.elapsed_ms(e0, e1) * 1e-3) / 1e9, 1)
    # the same kernel over 1 GiB in one launch (no launch gaps, no ramp between planes): the ceiling
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    for i in range(2):
        ekv.elitekv_stream_read(big, sink, stream=stream)
    ev.record(e0, stream)
    for i in range(10):
        ekv.elitekv_stream_read(big, sink, stream=stream)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    out["stream_read_GBs"] = max(round(10 * big.numel() / (ev.elapsed_ms(e0, e1) * 1e-3) / 1e9, 1),
                                 out["stream_read_planes_GBs"])
    # what the cache hint and the load path are worth: plain / non-temporal loads, into registers / straight into LDS
    kinds = {}
    for mode, name in ((0, "registers_plain"), (1, "registers_nt"), (2, "to_lds_plain"), (3, "to_lds_nt")):
        n_read = 0
        for i in range(2):
            n_read = ekv.elitekv_stream_read_mode(big, sink, mode, stream=stream)
        ev.record(e0, stream)
        for i in range(10):
            ekv.elitekv_stream_read_mode(big, sink, mode, stream=stream)
        ev.record(e1, stream)
        torch.cuda.synchronize()
        kinds[name] = round(10 * n_read / (ev.elapsed_ms(e0, e1) * 1e-3) / 1e9, 1)
    out["stream_read_1GiB_by_load_kind_GBs"] = kinds
    out["stream_read_GBs"] = max(out["stream_read_GBs"], *kinds.values())      # the ceiling: the best of them
    del big
    # a plain device-to-device copy of known size: the reference the HBM byte counters
    # (FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc) are scaled by
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev.record(e0, stream)
    for i in range(10):
        dst.copy_(src)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    out["copy_256MiB_GBs"] = round(10 * 2 * src.numel() / (ev.elapsed_ms(e0, e1) * 1e-3) / 1e9, 1)
    del src, dst

    # uncompressed cache: 2*n_h*d_h elements per token; use as many copies as fit ~2 GiB
    esz = 2 if cfg.dtype == "bf16" else 4
    full_bytes = B * S * 2 * n_h * d_h * esz
    n_full = max(2, min(4, (2 << 30) // full_bytes))
    g = torch.Generator(device=dev)
    g.manual_seed(1586)
    full = [(torch.randn(B * S, n_h, d_h, device=dev, dtype=torch.float32, generator=g).to(dt),
             torch.randn(B * S, n_h, d_h, device=dev, dtype=torch.float32, generator=g).to(dt))
            for _ in range(n_full)]
    o = torch.empty(B, n_h, d_h, dtype=dt, device=dev)
    ws = torch.empty(ekv.elitekv_mha_decode_workspace_bytes(dims, B, S, 0), dtype=torch.uint8, device=dev)
    for i in range(5):
        ekv.elitekv_mha_decode(dims, q_d, pos_d, seq_d, S, S, full[i % n_full][0], full[i % n_full][1], o, ws,
                               stream=stream)
    ev.record(e0, stream)
    for i in range(n):
        k_p, v_p = full[i % n_full]
        ekv.elitekv_mha_decode(dims, q_d, pos_d, seq_d, S, S, k_p, v_p, o, ws, stream=stream)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms = ev.elapsed_ms(e0, e1) / n
    out["mha_uncompressed_ms"] = round(ms, 5)
    out["mha_uncompressed_GBs"] = round(full_bytes / (ms * 1e-3) / 1e9, 1)
    out["mha_cache_bytes"] = full_bytes
    return out


def multiquery(ekv, ev, cfg, dims, planes, W_uk_d, W_uv_d, idx_d, dev, dt, stream, cache_bytes, T=8, iters=20):
    """A chunk of T queries per sequence (the last T positions, causal) over the same planes:
    every query consumes the sequence's cache rows; the rows come from HBM once and are re-used
    from the L2 of the XCD that the queries of a sequence share."""
    import torch
    B, S, n_h, d_h = cfg.batch, cfg.context, cfg.n_heads, cfg.head_dim
    if B * T > 65535:
        return None
    g = torch.Generator(device=dev)
    g.manual_seed(15861)
    q = torch.randn(B, T, n_h, d_h, device=dev, dtype=torch.float32, generator=g).to(dt)
    pos = (torch.arange(T, device=dev, dtype=torch.int32) + (S - T)).repeat(B)
    kv = pos + 1
    out = torch.empty(B, T, n_h, d_h, dtype=dt, device=dev)
    ws = torch.empty(ekv.elitekv_multiquery_workspace_bytes(dims, B, T, S, 0), dtype=torch.uint8, device=dev)

    def call(i):
        ke_p, c_p = planes[i % len(planes)]
        ekv.elitekv_multiquery_attn(dims, q, pos, kv, S, S, W_uk_d, W_uv_d, idx_d, ke_p, c_p, out, ws, stream=stream)
    for i in range(3):
        call(i)
    e0, e1 = ev.create(), ev.create()
    ev.record(e0, stream)
    for i in range(iters):
        call(i)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms = ev.elapsed_ms(e0, e1) / iters
    return {"queries_per_sequence": T, "ms_per_call": round(ms, 5), "us_per_query": round(ms * 1e3 / (B * T), 3),
            "cache_bytes_consumed_GBs": round(cache_bytes * T / (ms * 1e-3) / 1e9, 1),
            "query_tokens_per_s": round(B * T / (ms * 1e-3), 1)}


def block_step(ekv, ev, cfg, dims, planes, x_d, pos_d, slot_d, seq_d, W_ke_d, W_dkv_d, W_uk_d, W_uv_d, idx_d, dev, dt,
               stream, cache_bytes, args):
    """The whole attention block of the step (q = x W_q in front, W_o behind) in one call, next to
    the same work as torch matmuls around elitekv_decode_step."""
    import torch
    B, S, d, n_h, d_h = cfg.batch, cfg.context, cfg.d_model, cfg.n_heads, cfg.head_dim
    g = torch.Generator(device=dev)
    g.manual_seed(15863)
    W_q = (torch.randn(d, n_h, d_h, device=dev, dtype=torch.float32, generator=g) / d ** 0.5).to(dt)
    W_o = (torch.randn(n_h, d_h, d, device=dev, dtype=torch.float32, generator=g) / (n_h * d_h) ** 0.5).to(dt)
    y = torch.empty(B, d, dtype=dt, device=dev)
    out = torch.empty(B, n_h, d_h, dtype=dt, device=dev)
    ws = torch.empty(ekv.elitekv_block_step_workspace_bytes(dims, B, S, args.splits), dtype=torch.uint8, device=dev)
    sws = torch.empty(ekv.elitekv_decode_step_workspace_bytes(dims, B, S, args.splits), dtype=torch.uint8, device=dev)
    Wq2, Wo2 = W_q.reshape(d, n_h * d_h), W_o.reshape(n_h * d_h, d)
    n = max(20, args.steps // 2)

    def fused(i):
        ke_p, c_p = planes[i % len(planes)]
        ekv.elitekv_block_step(dims, x_d, pos_d, slot_d, seq_d, S, S, W_q, W_ke_d, W_dkv_d, W_uk_d, W_uv_d, W_o, idx_d,
                               ke_p, c_p, y, ws, n_splits=args.splits, stream=stream)

    def unfused(i):
        ke_p, c_p = planes[i % len(planes)]
        q = torch.matmul(x_d, Wq2).reshape(B, n_h, d_h)
        ekv.elitekv_decode_step(dims, x_d, q, pos_d, slot_d, seq_d, S, S, W_ke_d, W_dkv_d, W_uk_d, W_uv_d, idx_d, ke_p,
                                c_p, out, sws, n_splits=args.splits, stream=stream)
        torch.matmul(out.reshape(B, n_h * d_h), Wo2, out=y)

    res = {}
    e0, e1 = ev.create(), ev.create()
    for name, fn in (("ms_per_call", fused), ("ms_matmuls_around_decode_step", unfused)):
        for i in range(5):
            fn(i)
        ev.record(e0, stream)
        for i in range(n):
            fn(i)
        ev.record(e1, stream)
        torch.cuda.synchronize()
        res[name] = round(ev.elapsed_ms(e0, e1) / n, 5)
    weights = 2 * (2 * d * n_h * d_h + d * (2 * cfg.r * n_h + cfg.d_c) + cfg.d_c * n_h * (2 * d_h - 2 * cfg.r))
    res["algorithmic_bytes"] = cache_bytes + weights
    res["all_bytes_GBs"] = round((cache_bytes + weights) / (res["ms_per_call"] * 1e-3) / 1e9, 1)
    return res


def ropelite_search(ekv, ev, cfg, dev, stream, T=512, iters=3):
    """The greedy elite-chunk search of one layer (all heads, r rounds) on T sampled tokens."""
    import torch
    n_h, d_h, r = cfg.n_heads, cfg.head_dim, cfg.r
    g = torch.Generator(device=dev)
    g.manual_seed(15862)
    q = torch.randn(T, n_h, d_h, device=dev, dtype=torch.float32, generator=g)
    k = torch.randn(T, n_h, d_h, device=dev, dtype=torch.float32, generator=g)
    pos = torch.arange(T, dtype=torch.int32, device=dev)
    elite = torch.zeros(n_h, r, dtype=torch.int32, device=dev)
    ws = torch.empty(ekv.elitekv_ropelite_search_workspace_bytes(T, n_h, d_h, r), dtype=torch.uint8, device=dev)
    ekv.elitekv_ropelite_search(q, k, pos, r, cfg.rope_base, elite, None, ws, stream=stream)
    e0, e1 = ev.create(), ev.create()
    ev.record(e0, stream)
    for _ in range(iters):
        ekv.elitekv_ropelite_search(q, k, pos, r, cfg.rope_base, elite, None, ws, stream=stream)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms = ev.elapsed_ms(e0, e1) / iters
    evals = T * (T + 1) / 2 * n_h * r * (d_h // 2)      # (causal pair, chunk) evaluations over all rounds
    # Algorithm 1 per round, causal pair and chunk: the rotated and the plain 2-D dot product, their scaled
    # difference (8 flops), its share of the residual (1), and |residual - difference| added to the chunk's
    # distance (3): 12 fp32 flops.  The kernel takes the two dot products of a 16 x 16 tile of pairs as one
    # rank-4 fp32 MFMA per chunk (twice per round: once summed into the residual, once per candidate), the rest is
    # vector work; fp32 matrix and fp32 vector peak are the same 157.3 TFLOP/s on this chip, so the bound is
    # priced as "alu" against it
    tf = 12.0 * evals / (ms * 1e-3) / 1e12
    return {"tokens": T, "rounds": r, "ms_per_layer": round(ms, 4), "G_pair_chunk_evals_per_s": round(evals / ms / 1e6, 1),
            "bound": "alu", "flops_per_pair_chunk_round": 12, "TFLOPs": round(tf, 2), "peak_TFLOPs": FP32_VALU_PEAK_TFLOPS,
            "frac": round(tf / FP32_VALU_PEAK_TFLOPS, 4)}


def prefill_attn(ekv, ev, cfg, dims, planes, W_uk_d, W_uv_d, idx_d, dev, dt, stream, T=2048, iters=20):
    """Causal attention of a T-token prompt of one sequence over its own T cache rows (the step after
    the prefill-sized append): keys and values rebuilt once per row on the matrix cores, then flash
    attention.  Flops counted: the rebuild GEMM + 4 d_h per visible (query, key, head) pair."""
    import torch
    n_h, d_h, r, d_c = cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c
    ke_p, c_p = planes[0]
    T = int(min(T, c_p.shape[0]))
    g = torch.Generator(device=dev)
    g.manual_seed(15862)
    q = torch.randn(1, T, n_h, d_h, device=dev, dtype=torch.float32, generator=g).to(dt)
    pos = torch.arange(T, device=dev, dtype=torch.int32)
    kv = pos + 1
    out = torch.empty(1, T, n_h, d_h, dtype=dt, device=dev)
    d_ck = cfg.d_ck                                   # > 0: separated latents (W_uk_d = B^k_S, W_uv_d = B^v_S)
    nws = (ekv.elitekv_slrd_prefill_attn_workspace_bytes(dims, d_ck, 1, T, T) if d_ck
           else ekv.elitekv_prefill_attn_workspace_bytes(dims, 1, T, T))
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)

    def call():
        if d_ck:
            ekv.elitekv_slrd_prefill_attn(dims, d_ck, q, pos, kv, T, T, W_uk_d, W_uv_d, idx_d, ke_p, c_p, out, ws,
                                          stream=stream)
        else:
            ekv.elitekv_prefill_attn(dims, q, pos, kv, T, T, W_uk_d, W_uv_d, idx_d, ke_p, c_p, out, ws, stream=stream)
    for _ in range(3):
        call()
    e0, e1 = ev.create(), ev.create()
    ev.record(e0, stream)
    for _ in range(iters):
        call()
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms = ev.elapsed_ms(e0, e1) / iters
    fl_rebuild = (2.0 * T * n_h * (d_ck * (d_h - 2 * r) + (d_c - d_ck) * d_h) if d_ck
                  else 2.0 * T * d_c * n_h * (2 * d_h - 2 * r))
    fl_attn = 4.0 * d_h * n_h * (T * (T + 1) / 2)
    tf = (fl_rebuild + fl_attn) / (ms * 1e-3) / 1e12
    return {"tokens": T, "ms": round(ms, 5), "TFLOPs": round(tf, 1), "bound": "mfma", "peak_TFLOPs": 2500.0,
            "frac": round(tf / 2500.0, 4), "rebuild_GFLOP": round(fl_rebuild / 1e9, 1),
            "attention_GFLOP": round(fl_attn / 1e9, 1),
            "absorbed_form_GFLOP": round(n_h * (2.0 * (d_ck or d_c) + 2.0 * (d_c - d_ck if d_ck else d_c) + 4 * r)
                                         * (T * (T + 1) / 2) / 1e9, 1),
            "query_tokens_per_s": round(T / (ms * 1e-3), 1)}


def append_prefill(ekv, ev, cfg, dims, W_ke_d, W_dkv_d, W_dkv2_d, idx_d, dev, dt, stream, T=2048, iters=20):
    """The prefill-sized append of the same shape (a dense contraction on the matrix cores):
    T tokens through x [W_ke | W_dkv] + selective RoPE into fresh cache rows."""
    import torch
    d, n_h, r, d_c = cfg.d_model, cfg.n_heads, cfg.r, cfg.d_c
    g = torch.Generator(device=dev)
    g.manual_seed(15860)
    x = torch.randn(T, d, device=dev, dtype=torch.float32, generator=g).to(dt)
    pos = torch.arange(T, dtype=torch.int32, device=dev)
    slot = torch.arange(T, dtype=torch.int64, device=dev)
    ke = torch.zeros(T, n_h, 2 * r, dtype=dt, device=dev)
    c = torch.zeros(T, d_c, dtype=dt, device=dev)
    ws = torch.empty(16, dtype=torch.uint8, device=dev)      # appends of more than 64 tokens need no workspace

    def call():
        if cfg.d_ck:
            ekv.elitekv_slrd_append(dims, cfg.d_ck, x, pos, slot, W_ke_d, W_dkv_d, W_dkv2_d, idx_d, ke, c, ws=ws,
                                    stream=stream)
        else:
            ekv.elitekv_append(dims, x, pos, slot, W_ke_d, W_dkv_d, idx_d, ke, c, ws=ws, stream=stream)
    for _ in range(3):
        call()
    e0, e1 = ev.create(), ev.create()
    ev.record(e0, stream)
    for _ in range(iters):
        call()
    ev.record(e1, stream)
    torch.cuda.synchronize()
    ms = ev.elapsed_ms(e0, e1) / iters
    flops = 2.0 * T * d * (2 * r * n_h + d_c)
    tf = flops / (ms * 1e-3) / 1e12
    return {"tokens": T, "ms": round(ms, 5), "TFLOPs": round(tf, 1), "bound": "mfma", "peak_TFLOPs": 2500.0,
            "frac": round(tf / 2500.0, 4), "tokens_per_s": round(T / (ms * 1e-3), 1)}


def cpu_baseline(cfg, idx_h, W_ke_d, W_dkv_d, W_dkv2_d, W_uk_d, W_uv_d, q_d, x_d, host_planes0, cache_bytes):
    """The float64 oracle, as it stands, on the host's cores, over a bounded sample of the same
    workload: the append of the batch's tokens plus decode attention for a subset of heads of
    batch row 0, scaled linearly to all heads and rows."""
    import numpy as np
    import torch
    from oracle import elitekv_oracle as orc
    B, S, n_h, d_h = cfg.batch, cfg.context, cfg.n_heads, cfg.head_dim
    to64 = lambda t: t.detach().to("cpu").to(torch.float64).numpy()
    Wuk, Wuv, q = to64(W_uk_d), to64(W_uv_d), to64(q_d)
    ke0 = host_planes0[0][:S].to(torch.float64).numpy()
    c0 = host_planes0[1][:S].to(torch.float64).numpy()
    t0 = time.perf_counter()
    if cfg.d_ck:
        orc.slrd_append(to64(x_d), np.full(B, S - 1), to64(W_ke_d), to64(W_dkv_d), to64(W_dkv2_d), idx_h, d_h,
                        cfg.rope_base)
    else:
        orc.append(to64(x_d), np.full(B, S - 1), to64(W_ke_d), to64(W_dkv_d), idx_h, d_h, cfg.rope_base)
    t_app = time.perf_counter() - t0
    # decode: groups of 8 heads of batch row 0 (every batch row has the same shape and length),
    # one group after the other, round and round, until about 12 s of CPU time are spent
    groups = [list(range(h0, min(h0 + 8, n_h))) for h0 in range(0, n_h, 8)]
    budget, spent, done_heads, gi = 12.0, 0.0, 0, 0
    while spent < budget:
        heads = groups[gi % len(groups)]
        t0 = time.perf_counter()
        if cfg.d_ck:
            orc.slrd_decode_attn(q[:1], [S - 1], [ke0], [c0[:, :cfg.d_ck]], [c0[:, cfg.d_ck:]], [S], Wuk, Wuv, idx_h,
                                 d_h, cfg.rope_base, heads=heads)
        else:
            orc.decode_attn(q[:1], [S - 1], [ke0], [c0], [S], Wuk, Wuv, idx_h, d_h, cfg.rope_base, heads=heads)
        spent += time.perf_counter() - t0
        done_heads += len(heads)
        gi += 1
    est = t_app + spent / done_heads * n_h * B
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    return {"value": round(cache_bytes / est / 1e9, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "tokens_per_s": round(B / est, 4), "est_seconds_per_step": round(est, 3),
            "sample": "oracle append of %d token(s), timed once, + %.1f s of oracle decode over all %d cached tokens of "
                      "batch row 0 (%d head-decodes in groups of 8 heads), scaled to %d heads x %d batch rows "
                      "(host has %d logical cores)" % (B, spent, S, done_heads, n_h, B, os.cpu_count())}


if __name__ == "__main__":
    main()
