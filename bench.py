#!/usr/bin/env python3
"""Benchmark of the KIVI decode-attention hot path on one MI355X.

A step is one decode step at the workload's state: append the new token's key/value to the fp16
residual window, run the flush check, and run decode attention over the mixed-precision cache
(all through the C ABI).  Inputs are seeded synthetic tensors shaped like the paper's
Llama-2 / Mistral layers and are resident in HBM before the timed region.  The cache is
replicated `--copies` times and steps rotate over the copies so that every step streams its
cache from HBM rather than from the 256 MB Infinity Cache ("cold"); the same-copy ("warm")
figure is reported beside it.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(workload: str, path: str):
    """HBM bytes per decode-attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by
    what a plain copy of known size reads on the same counters.  The figures are not measured here:
    they are read from profiles/hbm_traffic.txt, which is rewritten whenever the counters are
    collected again for a changed kernel (lines `<workload> <path> <bytes> <kernel revision>`).
    None when the file has no line for this workload and path."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and not line.startswith("#") and parts[0] == workload and parts[1] == path:
                    return float(parts[2])
    except OSError:
        pass
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500,
                    help="untimed steps run before the timed ones, after the clocks have settled")
    ap.add_argument("--roofline-launches", type=int, default=2000,
                    help="launches of the attention-only loop the roofline figure is timed over (its own count, "
                         "independent of --steps)")
    ap.add_argument("--settle-seconds", type=float, default=0.3,
                    help="least duration of the untimed phase that lets the clocks settle")
    ap.add_argument("--workload", default="llama7b", choices=["tiny", "llama7b", "stream", "llama13b_4bit", "mistral_gqa"])
    ap.add_argument("--path", default="auto", choices=["auto", "valu", "mfma", "mfma1", "mfma2"])
    ap.add_argument("--copies", type=int, default=5)
    ap.add_argument("--cap-pad", type=int, default=1, help="spare 32-token tiles of quantised capacity")
    ap.add_argument("--cap-r-pad", type=int, default=0, help="spare 32-token tiles of residual-ring capacity")
    ap.add_argument("--skew", type=int, default=None,
                    help="byte offset between the cache arrays inside their allocations (default: the binding's)")
    ap.add_argument("--context", type=int, default=0, help="override the workload's context length (scaling studies)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    return ap.parse_args()


def cpu_baseline(w, k, v, q, seconds):
    """Time the oracle's decode attention (as it stands) on a bounded sample of kv-heads: half of
    the time budget with the numerical library's thread pool as it comes (all host cores it
    uses), half limited to one thread."""
    import numpy as np
    from oracle import kivi_oracle as ko
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        threads = 1
    n_q, n_r = w.split_single_step()
    rep = w.q_per_kv
    heads = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]

    def sample(budget):
        # Units are walked in order, pass after pass over the batch, until `budget` seconds of oracle
        # time are spent (one pass of a small workload takes about a second: too short a sample on
        # a busy host).
        done, t_total = 0, 0.0
        while t_total < budget:
            for (b, h) in heads:
                kk, vv = k[b:b + 1, h:h + 1], v[b:b + 1, h:h + 1]
                kq = ko.quantize_key(kk[:, :, :n_q], w.bits, w.group)       # setup, not timed
                vq = ko.quantize_value(vv[:, :, :n_q], w.bits, w.group)
                qq = q[b:b + 1, h * rep:(h + 1) * rep]
                t0 = time.perf_counter()
                ko.decode_attention(qq, kq, kk[:, :, n_q:], vq, vv[:, :, n_q:], w.group, w.softmax_scale)
                t_total += time.perf_counter() - t0
                done += 1
                if t_total >= budget:
                    break
        return done, t_total

    done, t_total = sample(seconds / 2)
    per_step = t_total / done * len(heads)
    result = {"value": w.batch / per_step, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
              "sample": f"decode attention of {done} (batch, kv-head) units ({done / len(heads):.1f} passes over the "
                        f"{len(heads)} units of the same workload), {t_total:.1f} s of oracle time, scaled to one pass; "
                        f"`cores` = threads of the numerical library's pool"}
    if threadpool_limits is not None and threads > 1:
        with threadpool_limits(limits=1):
            done1, t1 = sample(seconds / 2)
        result["single_thread"] = {"value": w.batch / (t1 / done1 * len(heads)), "unit": "tokens/s", "cores": 1,
                                   "sample": f"{done1} units, {t1:.1f} s, pool limited to one thread"}
    return result


def run_stream(args, w, path_name, path):
    """Streaming workload: prefill `prompt` tokens, then `decode_steps` single-token steps through
    kivi_decode_step (append, flush of one group every G steps, attention).  One untimed pass of all
    steps, then the same steps timed; a step here is one of the workload's decode steps, so --steps
    and --warmup are fixed to the workload's step count."""
    import numpy as np
    import torch
    from paper_2402_02750_amd import kivi, workloads

    total = w.prompt + w.decode_steps
    k, v = workloads.keys(w, total), workloads.values(w, total)
    kt, vt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    del k, v
    qs = torch.from_numpy(np.stack([workloads.queries(w, s) for s in range(w.decode_steps)])).cuda()
    k_new = [kt[:, :, w.prompt + s].contiguous() for s in range(w.decode_steps)]
    v_new = [vt[:, :, w.prompt + s].contiguous() for s in range(w.decode_steps)]
    cap_q = (total + 31) // 32 * 32
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, cap_q,
                              w.residual + w.group + 32 + 32 * args.cap_r_pad, decode_path=path)
    cache = kivi.Cache(layout, skew=args.skew)
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    marks = [torch.cuda.Event(enable_timing=True) for _ in range(w.decode_steps + 1)]

    def one_pass(mark_steps=False):
        cache.c.n_kq = cache.c.n_vq = cache.c.n_kr = cache.c.n_vr = 0
        kivi.kivi_prefill(layout, kt, vt, w.prompt, cache)
        bytes_total, flush_steps = 0, []
        marks[0].record(stream)
        for s in range(w.decode_steps):
            before = cache.c.n_kq
            kivi.kivi_decode_step(layout, cache, k_new[s], v_new[s], qs[s], w.softmax_scale, out,
                                  kivi.KIVI_FLUSH_WINDOW, stream)
            if mark_steps or s == w.decode_steps - 1:
                marks[s + 1].record(stream)
            if cache.c.n_kq != before:
                flush_steps.append(s)
            bytes_total += w.algorithmic_bytes(cache.c.n_kq, cache.c.n_kr)["all"]
        torch.cuda.synchronize()
        per_step = [marks[s].elapsed_time(marks[s + 1]) for s in range(w.decode_steps)] if mark_steps else None
        return marks[0].elapsed_time(marks[w.decode_steps]), bytes_total, flush_steps, per_step

    # untimed passes until the clocks have settled (two consecutive passes within 1 %, at least
    # --settle-seconds, at most 3 s), then the timed pass
    t_settle, prev_ms = time.perf_counter(), None
    while True:
        ms = one_pass()[0]
        elapsed = time.perf_counter() - t_settle
        if (prev_ms is not None and abs(ms - prev_ms) <= 0.01 * prev_ms and elapsed >= args.settle_seconds) or elapsed > 3.0:
            break
        prev_ms = ms
    ms, bytes_total, flush_steps, _ = one_pass()                 # the timed pass: events at its two ends only
    per_step = one_pass(mark_steps=True)[3]                      # once more with an event after every step
    flushes = len(flush_steps)
    flush_ms = [per_step[s] for s in flush_steps]
    plain_ms = [per_step[s] for s in range(w.decode_steps) if s not in set(flush_steps)]
    achieved = bytes_total / (ms * 1e-3) / 1e9
    return {
        "metric": "decode-attn tokens/s over 2-bit KV; achieved HBM GB/s vs MI355X peak",
        "value": w.batch * w.decode_steps / (ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": w.decode_steps, "warmup": w.decode_steps,
        "ms_per_step": ms / w.decode_steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": f"u{w.bits} codes, fp16 scale/zero/residual, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_q_heads} q-heads / {w.n_kv_heads} kv-heads, head_dim 128, "
                               f"prompt {w.prompt} + {w.decode_steps} decode steps, {w.bits}-bit, G=32, R={w.residual}, "
                               f"{flushes} flushes of one group",
                   "decode_path": path_name,
                   "attention_launches": kivi.kivi_decode_plan(layout, cache).launches,
                   "step": "kivi_decode_step: append newest token + flush (every 32nd step) + decode attention"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name, path_name),
                     "kernel": "whole steps (attention kernel plus, on flush steps, the copy and quantise kernels): "
                               "sum of the attention's algorithmic bytes over the steps / time of all steps",
                     "algorithmic_bytes_per_launch": bytes_total / w.decode_steps},
        "extra": {"flush_steps": flushes,
                  "ms_per_flush_step": sum(flush_ms) / max(len(flush_ms), 1),
                  "ms_per_step_without_flush": sum(plain_ms) / max(len(plain_ms), 1),
                  "note": "per-step times between HIP events recorded after every step of the timed pass; a flush "
                          "step appends, quantises one group of keys and values out of the rings and runs the attention"},
    }


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the units of work are independent (batch, kv-head) pairs: shard those).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2402_02750_amd import kivi, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    kivi.load_library()
    torch.cuda.set_device(0)
    w = workloads.CONFIGS[args.workload]
    if w.decode_steps:
        path = {"auto": kivi.KIVI_DECODE_AUTO, "valu": kivi.KIVI_DECODE_VALU, "mfma": kivi.KIVI_DECODE_MFMA,
            "mfma1": kivi.KIVI_DECODE_MFMA_ONE, "mfma2": kivi.KIVI_DECODE_MFMA_TWO}[args.path]
        print(json.dumps(run_stream(args, w, args.path, path)))
        return
    if args.context:
        w = workloads.scaled(w, name=f"{w.name}@{args.context}", context=args.context)
    n_q, n_r = w.split_single_step()
    L = w.context
    path = {"auto": kivi.KIVI_DECODE_AUTO, "valu": kivi.KIVI_DECODE_VALU, "mfma": kivi.KIVI_DECODE_MFMA,
            "mfma1": kivi.KIVI_DECODE_MFMA_ONE, "mfma2": kivi.KIVI_DECODE_MFMA_TWO}[args.path]

    k = workloads.keys(w, L)
    v = workloads.values(w, L)
    q = workloads.queries(w)
    kt, vt, qt = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), torch.from_numpy(q).cuda()
    cap_q = (n_q + 31) // 32 * 32 + 32 * args.cap_pad
    cap_r = w.residual + w.group + 32 + 32 * args.cap_r_pad
    layout = kivi.make_layout(w.batch, w.n_q_heads, w.n_kv_heads, w.bits, w.residual, max(cap_q, 32), cap_r,
                              decode_path=path)
    stream = torch.cuda.current_stream()

    # prefill (quantisation) -- timed separately, it is set-up for the decode step
    caches = [kivi.Cache(layout, skew=args.skew) for _ in range(max(args.copies, 1))]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kivi.kivi_prefill(layout, kt, vt, L, caches[0])          # warm-up of the quantise kernels
    caches[0].c.n_kq = caches[0].c.n_vq = caches[0].c.n_kr = caches[0].c.n_vr = 0
    ev0.record(stream)
    for c in caches:
        kivi.kivi_prefill(layout, kt, vt, L, c)
    ev1.record(stream)
    torch.cuda.synchronize()
    prefill_ms = ev0.elapsed_time(ev1) / len(caches)
    assert (caches[0].c.n_kq, caches[0].c.n_kr) == (n_q, n_r)
    k_new = kt[:, :, L - 1].contiguous()
    v_new = vt[:, :, L - 1].contiguous()
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")

    def step(c):
        # one decoding step: the newest token is (re-)appended as the last residual token, the flush
        # check runs, then attention -- kivi_decode_step does all three (one launch when no flush is due)
        c.c.n_kr -= 1
        c.c.n_vr -= 1
        kivi.kivi_decode_step(layout, c, k_new, v_new, qt, w.softmax_scale, out, kivi.KIVI_FLUSH_WINDOW, stream)

    def timed(n_steps, rotate, attention_only):
        """Average GPU time per iteration between two events on the launch stream; also the host's
        time per iteration to enqueue them (if that came close to the GPU time the launches would
        not be back to back)."""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(stream)
        for i in range(n_steps):
            c = caches[i % len(caches)] if rotate else caches[0]
            if attention_only:
                kivi.kivi_decode_attention(layout, c, qt, w.softmax_scale, out, stream)
            else:
                step(c)
        ev1.record(stream)
        enqueue_ms = (time.perf_counter() - t0) * 1e3
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / n_steps, enqueue_ms / n_steps

    # Clocks first, independently of --warmup: untimed blocks of 200 steps until two consecutive
    # blocks agree within 1 % and --settle-seconds have passed (at most 3 s).
    t_settle, prev_ms, settle_blocks = time.perf_counter(), None, 0
    while True:
        ms, _ = timed(200, rotate=True, attention_only=False)
        settle_blocks += 1
        elapsed = time.perf_counter() - t_settle
        if (prev_ms is not None and abs(ms - prev_ms) <= 0.01 * prev_ms and elapsed >= args.settle_seconds) or elapsed > 3.0:
            break
        prev_ms = ms

    def measure():
        for i in range(args.warmup):
            step(caches[i % len(caches)])
        cold_step_ms, enqueue_ms = timed(args.steps, rotate=True, attention_only=False)      # EXACTLY --steps steps
        warm_step_ms, _ = timed(max(args.steps, 200), rotate=False, attention_only=False)
        # the dominant kernel alone: back-to-back decode-attention launches (one kernel per launch in the
        # single-launch form), cold = rotating over the cache copies; its own launch count
        cold_attn_ms, _ = timed(args.roofline_launches, rotate=True, attention_only=True)
        warm_attn_ms, _ = timed(args.roofline_launches, rotate=False, attention_only=True)
        return cold_step_ms, enqueue_ms, warm_step_ms, cold_attn_ms, warm_attn_ms

    cold_step_ms, enqueue_ms, warm_step_ms, cold_attn_ms, warm_attn_ms = measure()
    # A step contains the attention launch: the launch alone cannot take longer than the step.  If the
    # two loops disagree by more than 2 % (clocks moved between them), measure once more.
    remeasured = False
    if cold_attn_ms > cold_step_ms * 1.02:
        remeasured = True
        cold_step_ms, enqueue_ms, warm_step_ms, cold_attn_ms, warm_attn_ms = measure()
    consistent = cold_attn_ms <= cold_step_ms * 1.02

    # The same launch dispatched one at a time (queue idle before it, two events around it): launch
    # latency, the event pair and the start from an idle device are all inside this figure, so it is
    # an upper bound for a single dispatch and not the kernel's rate; reported beside the
    # back-to-back figure for comparison with per-kernel durations of a trace.
    isolated = []
    for i in range(40):
        torch.cuda.synchronize()
        ev0.record(stream)
        kivi.kivi_decode_attention(layout, caches[i % len(caches)], qt, w.softmax_scale, out, stream)
        ev1.record(stream)
        torch.cuda.synchronize()
        isolated.append(ev0.elapsed_time(ev1) * 1e3)
    isolated_us = sorted(isolated)[len(isolated) // 2]

    # Yardstick: the library's plain read-only stream kernel on this machine -- over as many bytes as
    # one attention launch moves (rotating over different buffers, so cold like the launches above)
    # and over 1 GiB (where launch and ramp-up no longer matter).
    def stream_rate(n_bytes, n_bufs, iters):
        bufs = [torch.empty(n_bytes, dtype=torch.uint8, device="cuda").fill_(1) for _ in range(n_bufs)]
        sink = torch.empty(4096, dtype=torch.int32, device="cuda")
        for i in range(3):
            kivi.kivi_stream_read_probe(bufs[i % n_bufs], sink, stream)
        torch.cuda.synchronize()
        ev0.record(stream)
        for i in range(iters):
            kivi.kivi_stream_read_probe(bufs[i % n_bufs], sink, stream)
        ev1.record(stream)
        torch.cuda.synchronize()
        return n_bytes / (ev0.elapsed_time(ev1) / iters * 1e-3) / 1e9

    launch_bytes = w.algorithmic_bytes(n_q, n_r)["all"] // 16 * 16
    stream_same_size = stream_rate(launch_bytes, 5, 200)
    stream_1gib = stream_rate(1 << 30, 2, 20)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    bytes_ = w.algorithmic_bytes(n_q, n_r)
    achieved = bytes_["all"] / (cold_attn_ms * 1e-3) / 1e9
    achieved_packed = bytes_["packed"] / (cold_attn_ms * 1e-3) / 1e9
    result = {
        "metric": "decode-attn tokens/s over 2-bit KV; achieved HBM GB/s vs MI355X peak",
        "value": w.batch / (cold_step_ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": cold_step_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": f"u{w.bits} codes, fp16 scale/zero/residual, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, {w.n_q_heads} q-heads / {w.n_kv_heads} kv-heads, "
                               f"head_dim 128, context {L} = {n_q} quantised ({w.bits}-bit, G=32) + {n_r} fp16 residual",
                   "decode_path": args.path, "cache_copies_rotated": len(caches),
                   "attention_launches": kivi.kivi_decode_plan(layout, caches[0]).launches,
                   "step": "kivi_decode_step: append newest token + flush check + decode attention"},
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": measured_traffic(w.name, args.path),
            "kernel": "kivi_decode_attention: back-to-back launches between two HIP events on the launch stream, rotating cache copies (cold)",
            "algorithmic_bytes_per_launch": bytes_["all"],
            "achieved_packed_only": achieved_packed,
            "frac_packed_only": achieved_packed / HBM_PEAK_GBS,
            "launch_us": cold_attn_ms * 1e3,
            "launches_timed": args.roofline_launches,
            "launch_us_one_at_a_time": isolated_us,
            "consistent_with_ms_per_step": consistent,
            "stream_read_GBs_same_bytes": stream_same_size,
            "stream_read_GBs_1GiB": stream_1gib,
            "frac_of_stream_same_bytes": achieved / stream_same_size,
        },
        "extra": {
            "warm_ms_per_step": warm_step_ms, "warm_attn_us": warm_attn_ms * 1e3,
            "warm_achieved_GBs": bytes_["all"] / (warm_attn_ms * 1e-3) / 1e9,
            "host_enqueue_ms_per_step": enqueue_ms,
            "settle_blocks_of_200_steps": settle_blocks, "remeasured": remeasured,
            "prefill_quantize_ms": prefill_ms,
            "prefill_GBs": (2 * k.nbytes + bytes_["packed"] + bytes_["residual"]) / (prefill_ms * 1e-3) / 1e9,
        },
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, k, v, q, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
