#!/usr/bin/env python3
"""Benchmark of the VeriCache hot path on one MI355X.

Workload: config 2 of the five synthetic workloads (Llama-3-8B attention layer shape, 32 q / 8 KV heads, head_dim 128,
batch 16, context 65536; int4 g32 and int2 g64 block records of the same bf16 KV; verify window 32;
greedy accept over planted fp32 logits).  All inputs are seeded, synthetic and resident in HBM
before the timed region starts.

One step = one speculation round per compressor variant of that batch:
    A0  kept-index lists from the dropped-index lists (token-drop variant, 10 % budget)
    for s in 0..31 (the draft horizon; the bf16 tail holds the s tokens drafted so far):
        D1  draft attention over the retained bf16 rows (gather) + tail
        D2  draft attention over the int4 records + tail
        D3  draft attention over the int2 records + tail
    V1  verify attention of the 32 drafted positions over the full bf16 KV
    G1  greedy accept
`value` is the aggregate draft-attention bandwidth: algorithmic bytes of all D1+D2+D3 calls
divided by their summed HIP-event durations.  The swap-in leg (full KV from pinned host memory on
the copy stream, overlapped with int4 drafting) is measured outside the timed steps and reported
under "swap"; it never enters `value`.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--batch", type=int, default=16, help="sequences (config 2: 16)")
    ap.add_argument("--ctx", type=int, default=65536, help="context tokens (config 2: 65536)")
    ap.add_argument("--window", type=int, default=32)
    ap.add_argument("--vocab", type=int, default=128256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-swap", action="store_true")
    ap.add_argument("--no-compressor", action="store_true", help="skip the compress / decompress / top-k legs")
    ap.add_argument("--no-round3", action="store_true",
                    help="skip the config-3 round (32 layers, ctx 131072, 64-token horizon; pins 17 GB of host memory)")
    ap.add_argument("--round3", action="store_true", help="run the config-3 round even with --only")
    ap.add_argument("--no-small", action="store_true", help="skip the legs of workload configs 0 and 1")
    ap.add_argument("--no-config4", action="store_true", help="skip the ragged mixed batch (config 4)")
    ap.add_argument("--config4", action="store_true", help="run the ragged mixed batch even with --only")
    ap.add_argument("--only", default="", help="comma list of legs to run per step: keep,d1,d2,d3,verify,accept")
    ap.add_argument("--verify-series", action="store_true",
                    help="also time the verify kernel launch by launch under different preludes (back to back, after an "
                         "idle gap, between draft calls): shows how the clock management of the GPU shapes its timing")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def device_clocks():
    """Clock lines of rocm-smi (clocks cannot be pinned here; logged beside the figures), or None."""
    import subprocess
    try:
        r = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20)
        lines = [l.strip() for l in r.stdout.splitlines() if "clk" in l.lower() and "GPU[0]" in l]
        return [l for l in lines if any(k in l for k in ("sclk", "mclk", "fclk"))] or None
    except Exception:
        return None


TRAFFIC_PROFILE = os.path.join("profiles", "hbm_traffic_config2_round.txt")


def profile_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary: the table row
    'kernel  FETCH KiB  scaled MB  WRITE KiB  scaled MB ...' -> (read + written bytes, source), or
    (None, None) when the file or the row is missing."""
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_PROFILE)):
            f = line.split()
            if len(f) >= 5 and f[0] == kernel:
                return (float(f[2]) + float(f[4])) * 1e6, f"{TRAFFIC_PROFILE} (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not measured in this run)"
    except (OSError, ValueError):
        pass
    return None, None


def draft_bytes(n_seqs, hq, hkv, *, blocks=0, kept=0, tail=0):
    """Algorithmic bytes of one draft call: records + retained rows + index + tail + q + out."""
    per_head = blocks * 5120 + kept * (512 + 4) + tail * 512
    return n_seqs * (hkv * per_head + 2 * hq * 128 * 2)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives or sharding between GPUs); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2605_17613_amd as vc
    from tests import synth

    vc.load()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ctx = vc.Context(0)
    B, N, W, HQ, HKV = args.batch, args.ctx, args.window, 32, 8
    legs = set(args.only.split(",")) if args.only else {"keep", "d1", "d2", "d3", "verify", "accept"}

    t_setup = time.time()
    keep_n = -(-N // 10)
    lay = synth.make_layer(synth.SEED_BASE + 2, dev, ctx_len=[N] * B, n_q_heads=HQ, n_kv_heads=HKV,
                           keep=[keep_n] * B, keep_first=64, keep_last=256, quant_bits=(4, 2),
                           win=[W] * B, vocab=args.vocab)
    torch.cuda.synchronize()
    print(f"[bench] inputs built in {time.time() - t_setup:.1f}s", file=sys.stderr, flush=True)

    # per-draft-step tails: step s sees the first s window tokens of every sequence (their K/V are
    # the drafted tokens' own), gathered once into per-step pools
    tails = []
    for s in range(W):
        if s == 0:
            tails.append(None)
            continue
        sel = torch.cat([torch.arange(int(lay.cu_win[b]), int(lay.cu_win[b]) + s, device=dev) for b in range(B)])
        tails.append((lay.k_win[sel].contiguous(), lay.v_win[sel].contiguous(),
                      torch.arange(0, (B + 1) * s, s, dtype=torch.int32, device=dev), s))

    out = torch.empty_like(lay.q)
    keep_out = torch.empty_like(lay.keep_idx)
    cu_keep_out = torch.empty_like(lay.cu_keep)

    def draft_kw(kind, s):
        kw = {}
        if kind == "d1":
            kw.update(pool_k=lay.k_full, pool_v=lay.v_full, cu_ctx=lay.cu_ctx, keep_idx=keep_out,
                      cu_keep=cu_keep_out, max_keep=keep_n, sum_keep=keep_n * B)
        else:
            bits = 4 if kind == "d2" else 2
            kw.update(blocks=lay.blocks[bits], cu_blk=lay.cu_blk[bits], max_blk=lay.max_blk[bits], bits=bits,
                      sum_blk=lay.max_blk[bits] * B)
        if tails[s] is not None:
            tk, tv, cu, n = tails[s]
            kw.update(tail_k=tk, tail_v=tv, cu_tail=cu, max_tail=n)
        return kw

    ws_need = max(vc.vc_draft_workspace_bytes(HQ, HKV, B, **draft_kw(k, W - 1)) for k in ("d1", "d2", "d3"))
    vargs = dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=N, max_win=W, sum_ctx=N * B)
    ws_need = max(ws_need, vc.vc_verify_workspace_bytes(HQ, HKV, B, total_win=B * W, **vargs))
    ws = torch.empty(ws_need, dtype=torch.uint8, device=dev)
    vout = torch.empty_like(lay.q_win)
    rows = lay.logits.shape[0]
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    amax = torch.empty(rows, dtype=torch.int32, device=dev)
    aws = torch.empty(vc.vc_accept_workspace_bytes(rows, args.vocab), dtype=torch.uint8, device=dev)

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(record, hooks=False):
        """One pass of the hot path; `record` collects (leg, start_event, end_event).  With
        `hooks` the library also records events around the main kernel of each attention call
        (a pass of its own after the timed steps: the extra events cost a few microseconds)."""
        def timed(name, fn, main_kernel=False, always_hook=False):
            if main_kernel and (hooks or always_hook):
                # a second pair of events, recorded by the library around its main kernel only
                # (record once first: torch creates the HIP event on first use)
                k0, k1 = ev(), ev()
                k0.record(); k1.record()
                vc.vc_time_main_kernel(ctx, k0, k1)
                record.append((name + "_kernel", k0, k1))
            e0, e1 = ev(), ev()
            e0.record()
            fn()
            e1.record()
            record.append((name, e0, e1))
        if "keep" in legs:
            timed("keep", lambda: vc.vc_keep_from_dropped(ctx, lay.dropped_idx, lay.cu_drop, lay.cu_ctx, HKV, N,
                                                          keep_out, cu_keep_out))
        for s in range(W):
            for kind in ("d1", "d2", "d3"):
                if kind in legs:
                    kw = draft_kw(kind, s)
                    timed(kind, lambda kw=kw: vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV,
                                                               workspace=ws, **kw), main_kernel=True)
        if "verify" in legs:
            timed("verify", lambda: vc.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale,
                                                      vout, n_seqs=B, workspace=ws, **vargs), main_kernel=True,
                  always_hook=True)      # one call per step: the kernel and the call are timed on the same launches
        if "accept" in legs:
            timed("accept", lambda: vc.vc_accept_len(ctx, lay.logits, lay.cu_rows, lay.draft_ids, lay.cu_win,
                                                     acc, nxt, amax, workspace=aws))

    if "keep" not in legs:   # d1 still needs kept lists
        vc.vc_keep_from_dropped(ctx, lay.dropped_idx, lay.cu_drop, lay.cu_ctx, HKV, N, keep_out, cu_keep_out)
    if args.calib_copy:
        # 1 GiB read + 1 GiB written by a plain elementwise kernel with 16-byte accesses per lane,
        # the same access width the library's kernels use (the derived counters price a 128-byte
        # request as 64 bytes, so the reference must issue the same kind of request)
        src = torch.zeros(1 << 29, dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step([])
    torch.cuda.synchronize()
    rec = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    rec_k = []
    for _ in range(args.steps):
        step(rec_k, hooks=True)
    torch.cuda.synchronize()

    dur = {}
    for name, e0, e1 in rec + [r for r in rec_k if r[0].endswith("_kernel") and r[0] != "verify_kernel"]:
        dur.setdefault(name, []).append(e0.elapsed_time(e1))
    # the draft calls of the pass that carried the library's kernel events (their call times include
    # the two extra event records; the kernel times are compared with THESE call times)
    for name, e0, e1 in rec_k:
        if name in ("d1", "d2", "d3"):
            dur.setdefault(name + "_hookpass", []).append(e0.elapsed_time(e1))
    mean_ms = {k: sum(v) / len(v) for k, v in dur.items()}

    def spread(name):
        """median and minimum of a leg's per-call times, microseconds"""
        v = sorted(dur[name])
        return {"median_us": v[len(v) // 2] * 1e3, "min_us": v[0] * 1e3, "calls": len(v)}

    # algorithmic bytes / flops per call
    tail_avg = (W - 1) / 2.0
    by = {
        "d1": draft_bytes(B, HQ, HKV, kept=keep_n, tail=tail_avg),
        "d2": draft_bytes(B, HQ, HKV, blocks=N // 32, tail=tail_avg),
        "d3": draft_bytes(B, HQ, HKV, blocks=N // 64, tail=tail_avg),
    }
    verify_flops = B * 4 * HQ * 128 * (W * N + W * (W + 1) / 2)
    verify_bytes = B * (2 * HKV * N * 256 + 2 * HKV * W * 256 + 2 * W * HQ * 256)
    accept_bytes = rows * args.vocab * 4
    res = {}
    tot_b, tot_t = 0.0, 0.0
    for k in ("d1", "d2", "d3"):
        if k in mean_ms:
            res[k] = {"us": mean_ms[k] * 1e3, "GBps": by[k] / (mean_ms[k] * 1e-3) / 1e9,
                      "frac_hbm": by[k] / (mean_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                      "kernel_us": mean_ms[k + "_kernel"] * 1e3, "call_us_same_launches_as_kernel_us": mean_ms[k + "_hookpass"] * 1e3,
                      "kernel_frac_hbm": by[k] / (mean_ms[k + "_kernel"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, **spread(k)}
            tot_b += by[k] * len(dur[k])
            tot_t += sum(dur[k]) * 1e-3
    value = tot_b / tot_t / 1e9 if tot_t > 0 else 0.0
    if "verify" in mean_ms:
        tf = verify_flops / (mean_ms["verify"] * 1e-3) / 1e12
        ai = verify_flops / verify_bytes
        attainable = min(MFMA_BF16_PEAK_TFLOPS, ai * HBM_PEAK_GBPS / 1e3)
        res["verify"] = {"us": mean_ms["verify"] * 1e3, "kernel_us": mean_ms["verify_kernel"] * 1e3, "TFLOPs": tf, "frac_mfma": tf / MFMA_BF16_PEAK_TFLOPS,
                         "frac_attainable": tf / attainable, "GBps": verify_bytes / (mean_ms["verify"] * 1e-3) / 1e9,
                         **spread("verify")}
    if "accept" in mean_ms:
        res["accept"] = {"us": mean_ms["accept"] * 1e3, "GBps": accept_bytes / (mean_ms["accept"] * 1e-3) / 1e9,
                         **spread("accept")}
    if "keep" in mean_ms:
        res["keep"] = {"us": mean_ms["keep"] * 1e3, **spread("keep")}

    # roofline of the dominant kernel of a round: the int4 record draft kernel (32 launches per
    # step against one verify); duration = HIP events the library records on the call's stream
    # right before and after that kernel (the merge/tail kernel of the call is not included; the
    # whole call is in legs.d2)
    roofline = None
    if "d2" in mean_ms:
        a = by["d2"] / (mean_ms["d2_kernel"] * 1e-3) / 1e9
        # HBM bytes per launch: not measurable from inside the process; read from the committed summary of
        # the rocprofv3 --pmc runs of this same command (FETCH_SIZE and WRITE_SIZE, each scaled by what the
        # counter reads for a copy kernel of known size), valid for the default config-2 sizes only
        traffic, traffic_src = (profile_traffic("draft_quant_kernel<4,4>") if (B, N, W) == (16, 65536, 32) else (None, None))
        roofline = {"bound": "hbm", "kernel": "draft_quant_kernel<4>", "achieved": a, "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": a / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_src,
                    "bytes_per_launch": by["d2"], "avg_us": mean_ms["d2_kernel"] * 1e3,
                    "call_us": mean_ms["d2"] * 1e3, "call_frac": by["d2"] / (mean_ms["d2"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                    "timed": "HIP events recorded by the library around draft_quant_kernel<4> on the call's stream"}

    series = None
    if args.verify_series and "verify" in legs and "d2" in legs:
        series = measure_verify_series(vc, ctx, torch, lambda: vc.vc_verify_attn(
            ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, vout, n_seqs=B, workspace=ws, **vargs),
            lambda: vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV, workspace=ws, **draft_kw("d2", 0)))

    swap = None
    if not args.no_swap and "d2" in legs:
        swap = measure_swap(vc, ctx, lay, torch, draft_kw, out, ws, HKV, N, B, W)

    comp = None
    if not args.no_compressor and not args.only:
        comp = measure_compressor(vc, ctx, lay, torch, HKV, N, B)

    loop32 = None
    if not args.no_compressor and not args.only:
        try:
            loop32 = measure_layer_loop(vc, ctx, lay, torch, HQ, HKV, N, B)
        except Exception as e:
            loop32 = {"error": f"{type(e).__name__}: {e}"}

    compact = None
    if not args.no_compressor and not args.only:
        try:
            compact = measure_compact_rows(vc, ctx, lay, torch, keep_out, HQ, HKV, B, keep_n, out, ws)
        except Exception as e:
            compact = {"error": f"{type(e).__name__}: {e}"}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(lay, torch, np, HQ, HKV, N)

    round3 = None
    ragged = None
    small = None
    if args.round3 or args.config4 or not ((args.no_round3 and args.no_config4 and args.no_small) or args.only):
        del lay, ws
        torch.cuda.empty_cache()
    if not (args.no_small or args.only):
        try:
            small = measure_small_configs(vc, ctx, torch)
        except Exception as e:
            small = {"error": f"{type(e).__name__}: {e}"}
        torch.cuda.empty_cache()
    if args.config4 or not (args.no_config4 or args.only):
        try:
            ragged = measure_config4(vc, ctx, torch)
        except Exception as e:
            ragged = {"error": f"{type(e).__name__}: {e}"}
        torch.cuda.empty_cache()
    if args.round3 or not (args.no_round3 or args.only):
        try:
            round3 = measure_round3(vc, ctx, torch)
        except Exception as e:      # the host may not have 17 GB to pin: the headline line must still be printed
            round3 = {"error": f"{type(e).__name__}: {e}"}

    line = {
        "metric": "draft_attn_hbm_GBps", "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16/int4/int2 inputs, fp16+bf16 MFMA, fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"config2: batch {B}, ctx {N}, 32q/8kv heads, d128, int4 g32 + int2 g64 + 10% token drop, "
                               f"window {W}, vocab {args.vocab}",
                   "step": f"keep-index + {W} draft steps x (bf16 gather, int4, int2) + verify + accept"},
        "legs": res,
        "verify_TFLOPs": res.get("verify", {}).get("TFLOPs"),
        "roofline": roofline, "verify_series": series, "swap": swap, "compressor": comp, "layer_loop": loop32, "compact_rows": compact, "config0_config1": small, "config3_round": round3, "config4_ragged": ragged,
        "clocks_after_run": device_clocks(),
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    ctx.close()


def measure_verify_series(vc, ctx, torch, verify, draft):
    """Verify call times, launch by launch (microseconds), under four preludes.  The kernel keeps the
    matrix cores, LDS and HBM busy at once; what the series show is the GPU's own clock management."""
    def clocks():
        c = device_clocks()
        return [l.split(":")[-1].strip() for l in c] if c else None

    def run(n, before=None):
        evs = []
        for _ in range(n):
            if before:
                before()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); verify(); e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        return [round(a.elapsed_time(b) * 1e3) for a, b in evs]

    def idle():
        torch.cuda.synchronize()
        time.sleep(0.005)

    torch.cuda.synchronize()
    time.sleep(1.0)
    res = {"clocks_idle": clocks()}
    res["back_to_back_after_1s_idle_us"] = run(16)
    res["clocks_after_back_to_back"] = clocks()
    res["back_to_back_again_us"] = run(12)
    res["after_32_int4_draft_calls_each_us"] = run(12, before=lambda: [draft() for _ in range(32)])
    res["after_5ms_idle_each_us"] = run(12, before=idle)
    return res


def measure_compact_rows(vc, ctx, lay, torch, keep_idx, HQ, HKV, B, keep_n, out, ws, reps=40):
    """The d1 leg's kept rows stored compactly - row r of a sequence's pool holds, for every KV head, that
    head's r-th kept token (all heads keep the same count) - and read through the contiguous path of
    vc_draft_attn: what a deployment that evicts the dropped tokens from HBM would hold.  Same rows, same
    bytes as d1 without its index lists; not part of `value`."""
    dev = lay.q.device
    idx = keep_idx.view(B, HKV, keep_n).long() + lay.cu_ctx[:-1].view(B, 1, 1).long()       # pool rows
    head = torch.arange(HKV, device=dev).view(1, HKV, 1)
    ck = lay.k_full[idx, head].permute(0, 2, 1, 3).reshape(B * keep_n, HKV, 128).contiguous()
    cv = lay.v_full[idx, head].permute(0, 2, 1, 3).reshape(B * keep_n, HKV, 128).contiguous()
    cu = torch.arange(0, (B + 1) * keep_n, keep_n, dtype=torch.int32, device=dev)
    kw = dict(pool_k=ck, pool_v=cv, cu_ctx=cu, max_keep=keep_n, sum_keep=keep_n * B)
    ref = torch.empty_like(out)
    vc.vc_draft_attn(ctx, lay.q, lay.scale, ref, n_kv_heads=HKV, workspace=ws, pool_k=lay.k_full, pool_v=lay.v_full,
                     cu_ctx=lay.cu_ctx, keep_idx=keep_idx, cu_keep=cu, max_keep=keep_n, sum_keep=keep_n * B)
    for _ in range(5):
        vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV, workspace=ws, **kw)
    torch.cuda.synchronize()
    same = bool(torch.equal(out.view(torch.int16), ref.view(torch.int16)))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV, workspace=ws, **kw)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    nbytes = draft_bytes(B, HQ, HKV, kept=keep_n, tail=0) - B * HKV * keep_n * 4      # no index lists
    return {"us": us, "GBps": nbytes / us / 1e3, "frac_hbm": nbytes / us / 1e3 / HBM_PEAK_GBPS,
            "same_bits_as_gather": same, "note": "kept rows stored compactly, contiguous path, no tail; back-to-back calls"}


def measure_layer_loop(vc, ctx, lay, torch, HQ, HKV, N, B, layers=32, reps=3):
    """int4 draft attention over `layers` distinct layers back to back (each layer its own records,
    43 GB at config-2 size, so that no cache level can hold a layer from one pass to the next):
    microseconds per layer call and the rate over the records."""
    dev = lay.k_full.device
    nb = lay.max_blk[4]
    blocks = torch.empty((layers,) + tuple(lay.blocks[4].shape), dtype=torch.uint8, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(20260518)
    k = torch.empty_like(lay.k_full)
    v = torch.empty_like(lay.v_full)
    for l in range(layers):
        k.copy_(torch.randn(k.shape, device=dev, dtype=torch.float32, generator=g))
        v.copy_(torch.randn(v.shape, device=dev, dtype=torch.float32, generator=g))
        vc.vc_compress_quant(ctx, k, v, lay.cu_ctx, lay.cu_blk[4], 4, nb, blocks[l])
    del k, v
    q = torch.randn((layers,) + tuple(lay.q.shape), device=dev, generator=g).to(torch.bfloat16)
    out = torch.empty_like(q)
    kw = dict(cu_blk=lay.cu_blk[4], max_blk=nb, bits=4, sum_blk=nb * B)
    ws = torch.empty(vc.vc_draft_workspace_bytes(HQ, HKV, B, blocks=blocks[0], **kw), dtype=torch.uint8, device=dev)

    def one_pass():
        for l in range(layers):
            vc.vc_draft_attn(ctx, q[l], lay.scale, out[l], n_kv_heads=HKV, workspace=ws, blocks=blocks[l], **kw)

    one_pass()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        one_pass()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (reps * layers)
    bytes_call = draft_bytes(B, HQ, HKV, blocks=N // 32)
    return {"layers": layers, "records_GB": blocks.numel() / 1e9, "us_per_layer_call": us,
            "GBps": bytes_call / us / 1e3, "frac_hbm": bytes_call / us / 1e3 / HBM_PEAK_GBPS}


def measure_compressor(vc, ctx, lay, torch, HKV, N, B, reps=5):
    """The compressor-side entry points on the same layer (not part of a step): bf16 KV -> int4 /
    int2 records, int4 records -> bf16 KV, kept lists (10 %) from fp32 scores.  GB/s counts the
    algorithmic bytes read plus written."""
    dev = lay.k_full.device
    res = {}

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    kv_bytes = 2 * B * N * HKV * 256
    for bits in (4, 2):
        ref = lay.blocks[bits]
        blocks = torch.empty_like(ref)
        nb = lay.max_blk[bits]
        ms = timed(lambda: vc.vc_compress_quant(ctx, lay.k_full, lay.v_full, lay.cu_ctx, lay.cu_blk[bits], bits, nb, blocks))
        res[f"compress_int{bits}"] = {"us": ms * 1e3, "GBps": (kv_bytes + blocks.numel()) / (ms * 1e-3) / 1e9,
                                      "equals_generator_records": bool(torch.equal(blocks, ref))}
        if bits == 4:
            ko, vo = torch.empty_like(lay.k_full), torch.empty_like(lay.v_full)
            ms = timed(lambda: vc.vc_decompress_quant(ctx, blocks, lay.cu_blk[bits], lay.cu_ctx, bits, nb, ko, vo))
            res["decompress_int4"] = {"us": ms * 1e3, "GBps": (kv_bytes + blocks.numel()) / (ms * 1e-3) / 1e9}
            del ko, vo
        del blocks
    # decode attention over the uncompressed bf16 KV (what drafting would cost without a compressor)
    HQ = lay.n_q_heads
    fkw = dict(pool_k=lay.k_full, pool_v=lay.v_full, cu_ctx=lay.cu_ctx, max_keep=N, sum_keep=N * B)
    fout = torch.empty_like(lay.q)
    fws = torch.empty(vc.vc_draft_workspace_bytes(HQ, HKV, B, **fkw), dtype=torch.uint8, device=dev)
    ms = timed(lambda: vc.vc_draft_attn(ctx, lay.q, lay.scale, fout, n_kv_heads=HKV, workspace=fws, **fkw))
    res["full_bf16_decode"] = {"us": ms * 1e3, "GBps": B * N * HKV * 512 / (ms * 1e-3) / 1e9}
    del fout, fws
    keep_n = N // 10
    g = torch.Generator(device=dev)
    g.manual_seed(20260517)
    scores = torch.randn(B * HKV * N, device=dev, dtype=torch.float32, generator=g)
    cu_keep = torch.arange(0, (B + 1) * keep_n, keep_n, dtype=torch.int32, device=dev)
    first = torch.full((B,), 64, dtype=torch.int32, device=dev)
    last = torch.full((B,), 256, dtype=torch.int32, device=dev)
    keep = torch.empty(B * HKV * keep_n, dtype=torch.int32, device=dev)
    ms = timed(lambda: vc.vc_topk_keep(ctx, scores, lay.cu_ctx, cu_keep, HKV, keep, forced_first=first, forced_last=last))
    res["topk_keep"] = {"us": ms * 1e3, "lists": B * HKV, "positions": N, "kept": keep_n,
                        "GBps": (scores.numel() * 4 + keep.numel() * 4) / (ms * 1e-3) / 1e9}
    del scores, keep
    # sampling-based acceptance on the round's logits: draft logits = verify logits + noise
    if lay.logits is not None:
        rows, vocab = lay.logits.shape
        tw = lay.draft_ids.numel()
        sel = torch.cat([torch.arange(int(lay.cu_rows[b]), int(lay.cu_rows[b]) + lay.win[b], device=dev) for b in range(B)])
        dlog = lay.logits[sel] + 0.3 * torch.randn((tw, vocab), device=dev, generator=g)
        ua = torch.rand(tw, device=dev, generator=g)
        ur = torch.rand(B, device=dev, generator=g)
        acc = torch.empty(B, dtype=torch.int32, device=dev)
        nxt = torch.empty(B, dtype=torch.int32, device=dev)
        sws = torch.empty(vc.vc_accept_sample_workspace_bytes(rows, tw, B, vocab), dtype=torch.uint8, device=dev)
        ms = timed(lambda: vc.vc_accept_sample(ctx, lay.logits, dlog, lay.cu_rows, lay.draft_ids, lay.cu_win, 0.8, ua, ur,
                                               acc, nxt, workspace=sws))
        res["accept_sample"] = {"us": ms * 1e3, "rows": rows + tw, "vocab": vocab,
                                "GBps": (rows + tw) * vocab * 4 / (ms * 1e-3) / 1e9,
                                "mean_accept_len": float(acc.float().mean())}
    return res


def measure_swap(vc, ctx, lay, torch, draft_kw, out, ws, HKV, N, B, W):
    """Full-KV reload of every sequence in 8192-token chunks on the copy stream, alone and
    overlapped with int4 drafting; overlap = (T_draft + T_swap - T_both) / min(T_draft, T_swap)."""
    dev = lay.k_full.device
    row_bytes = HKV * 128 * 2
    host_k = torch.empty(lay.k_full.shape, dtype=torch.bfloat16, pin_memory=True)
    host_v = torch.empty(lay.v_full.shape, dtype=torch.bfloat16, pin_memory=True)
    host_k.copy_(lay.k_full)
    host_v.copy_(lay.v_full)
    dst_k = torch.empty_like(lay.k_full)
    dst_v = torch.empty_like(lay.v_full)
    chunk_tok = 8192
    chunks = [(t * row_bytes, t * row_bytes, min(chunk_tok, B * N - t) * row_bytes) for t in range(0, B * N, chunk_tok)]
    total = 2 * B * N * row_bytes

    def swap_all():
        vc.vc_swap_in(ctx, host_k, dst_k, chunks)
        return vc.vc_swap_in(ctx, host_v, dst_v, chunks) + len(chunks) - 1

    def drafts(n):
        for i in range(n):
            vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV, workspace=ws, **draft_kw("d2", i % W))

    torch.cuda.synchronize()
    t0 = time.perf_counter(); swap_all(); vc.vc_swap_sync(ctx); t_swap = time.perf_counter() - t0
    ok = bool(torch.equal(dst_k[-4096:], lay.k_full[-4096:]) and torch.equal(dst_v[:4096], lay.v_full[:4096]))
    # enough draft steps to cover the copy
    drafts(4); torch.cuda.synchronize()
    t0 = time.perf_counter(); drafts(32); torch.cuda.synchronize(); t32 = time.perf_counter() - t0
    n_steps = max(32, int(math.ceil(t_swap / (t32 / 32))))
    t0 = time.perf_counter(); drafts(n_steps); torch.cuda.synchronize(); t_draft = time.perf_counter() - t0
    t0 = time.perf_counter()
    last = swap_all()
    drafts(n_steps)
    vc.vc_swap_wait(ctx, last)
    torch.cuda.synchronize()
    vc.vc_swap_sync(ctx)
    t_both = time.perf_counter() - t0

    # chunk-streamed verify through a staging ring (section 5.1: the in-flight KV): the full KV never
    # exists on the device; every 8192-token chunk lands in slot i mod R of a ring, is attended to as soon
    # as its ticket has landed, and slots are reloaded only after the range calls that read them have run
    # (vc_mark behind the range call, vc_swap_after before the reload).  The ring is reloaded in groups of
    # G chunks, one device-side wait per group: every cross-stream wait in front of a copy stalls the copy
    # engine for a fraction of a millisecond (measured for the 128 chunks, 79.0 ms of pure transfer:
    # G = 1, R = 3: 88.4 ms; G = 2: 91.0; G = 8, R = 16: 79.7 ms; G = 16: 79.7).
    # Exposed = from the moment the last chunk has landed to the end of the merge.
    streamed = None
    if N % chunk_tok == 0 and lay.q_win is not None:
        G = 8
        R = 2 * G
        ring_k = torch.empty((R * chunk_tok, HKV, 128), dtype=torch.bfloat16, device=dev)
        ring_v = torch.empty_like(ring_k)
        per_seq = N // chunk_tok
        nch = len(chunks)
        slot_of = []
        for i in range(nch):
            t = torch.zeros(B, dtype=torch.int32, device=dev)
            t[i // per_seq] = i % R
            slot_of.append(t)
        full = dict(k=dst_k, v=dst_v, cu_ctx=lay.cu_ctx, max_ctx=N, max_win=W, n_seqs=B, chunk_tokens=chunk_tok)
        ring = dict(k=ring_k, v=ring_v, cu_ctx=lay.cu_ctx, max_ctx=N, max_win=W, n_seqs=B, chunk_tokens=chunk_tok, ring_slots=R)
        vws = torch.empty(vc.vc_verify_workspace_bytes(lay.n_q_heads, HKV, B, total_win=B * W, k=dst_k, v=dst_v,
                                                       cu_ctx=lay.cu_ctx, max_ctx=N, max_win=W, chunk_tokens=chunk_tok),
                          dtype=torch.uint8, device=dev)
        vout = torch.empty_like(lay.q_win)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        vc.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, vout, workspace=vws, **full)
        torch.cuda.synchronize()
        t_verify = time.perf_counter() - t0
        ref = vout.clone()
        vout.zero_()
        chunk_bytes = chunk_tok * row_bytes

        def issue_group(g0):
            """chunks g0 .. g0 + G - 1 into their slots: K copies, then V copies; ticket of the last V copy of each"""
            idx = range(g0, min(nch, g0 + G))
            cs = [(chunks[i][0], (i % R) * chunk_bytes, chunks[i][2]) for i in idx]
            vc.vc_swap_in(ctx, host_k, ring_k, cs)
            first = vc.vc_swap_in(ctx, host_v, ring_v, cs)
            return {i: first + j for j, i in enumerate(idx)}

        e_landed, e_done = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tickets = {}
        tickets.update(issue_group(0))
        tickets.update(issue_group(G))
        for i in range(nch):
            vc.vc_swap_wait(ctx, tickets.pop(i))
            if i == nch - 1:
                e_landed.record()
            b, c = divmod(i, per_seq)
            vc.vc_verify_attn_range(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, b, b + 1, c * chunk_tok,
                                    (1 << 30) if c == per_seq - 1 else (c + 1) * chunk_tok, workspace=vws,
                                    ring_slot=slot_of[i], **ring)
            if (i + 1) % G == 0 and i + 1 + G < nch:
                # the group that just finished frees its G slots for the group after the one in flight
                vc.vc_swap_after(ctx, vc.vc_mark(ctx))
                tickets.update(issue_group(i + 1 + G))
        vc.vc_verify_finish(ctx, lay.cu_win, vout, n_q_heads=lay.n_q_heads, n_kv_heads=HKV, workspace=vws, ring_slot=slot_of[0], **ring)
        e_done.record()
        torch.cuda.synchronize()
        t_stream = time.perf_counter() - t0
        streamed = {"verify_alone_ms": t_verify * 1e3, "swap_then_verify_ms": (t_swap + t_verify) * 1e3,
                    "streamed_ms": t_stream * 1e3, "ring_slots": R, "chunks_per_reload_group": G, "ring_chunk_tokens": chunk_tok,
                    "device_staging_MB": 2 * ring_k.numel() * 2 / 1e6, "full_kv_MB": total / 1e6,
                    "exposed_after_last_chunk_ms": e_landed.elapsed_time(e_done),
                    "same_bits": bool(torch.equal(ref.view(torch.int16), vout.view(torch.int16)))}
        del ring_k, ring_v, vws
    # reload of the dropped rows only (token dropping keeps 10 % resident): the host holds them
    # packed; per sequence two contiguous copies into a staging buffer and a short placement kernel,
    # all on the copy stream, alone and under bf16-gather drafting
    rows = None
    if lay.dropped_idx is not None:
        nd = N - lay.max_keep
        rows_bytes = 2 * B * HKV * nd * 256
        pk = torch.empty((B * HKV * nd, 128), dtype=torch.bfloat16, device=dev)
        pv = torch.empty_like(pk)
        vc.vc_pack_rows(ctx, lay.k_full, lay.v_full, lay.dropped_idx, lay.cu_drop, lay.cu_ctx, HKV, nd, pk, pv)
        hpk = torch.empty(pk.shape, dtype=torch.bfloat16, pin_memory=True); hpk.copy_(pk)
        hpv = torch.empty(pv.shape, dtype=torch.bfloat16, pin_memory=True); hpv.copy_(pv)
        del pk, pv
        stage_k = torch.empty((HKV * nd, 128), dtype=torch.bfloat16, device=dev)
        stage_v = torch.empty_like(stage_k)
        cu_drop_host = lay.cu_drop.cpu()
        dst_k.fill_(float("nan")); dst_v.fill_(float("nan"))
        torch.cuda.synchronize()

        def rows_all():
            return vc.vc_swap_in_rows(ctx, hpk, hpv, stage_k, stage_v, dst_k, dst_v, lay.dropped_idx, lay.cu_drop,
                                      cu_drop_host, lay.cu_ctx, HKV, 0, B) + B - 1

        t0 = time.perf_counter(); rows_all(); vc.vc_swap_sync(ctx); t_rows = time.perf_counter() - t0
        # every dropped row arrived, every kept row is still untouched
        landed = ~torch.isnan(dst_k[:, :, 0].float())
        rows_ok = bool(int(landed.sum()) == B * HKV * nd and torch.equal(dst_k[landed], lay.k_full[landed]))

        def drafts1(n):
            for i in range(n):
                vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV, workspace=ws, **draft_kw("d1", i % W))

        drafts1(4); torch.cuda.synchronize()
        t0 = time.perf_counter(); drafts1(64); torch.cuda.synchronize(); t64 = time.perf_counter() - t0
        n1 = max(64, int(math.ceil(t_rows / (t64 / 64))))
        t0 = time.perf_counter(); drafts1(n1); torch.cuda.synchronize(); t_d1 = time.perf_counter() - t0
        t0 = time.perf_counter()
        last = rows_all()
        drafts1(n1)
        vc.vc_swap_wait(ctx, last)
        torch.cuda.synchronize()
        vc.vc_swap_sync(ctx)
        t_both1 = time.perf_counter() - t0
        rows = {"bytes": rows_bytes, "fraction_of_full": rows_bytes / total, "alone_ms": t_rows * 1e3,
                "GBps": rows_bytes / t_rows / 1e9, "draft_steps": n1, "draft_alone_ms": t_d1 * 1e3, "both_ms": t_both1 * 1e3,
                "overlap": (t_d1 + t_rows - t_both1) / min(t_d1, t_rows), "rows_ok": rows_ok}
    # the execution loop of section 5.2 for the 16 requests of this layer: the library's admission
    # control (Algorithm 1) staggers their reloads and verifies; iterations are not clocked, so a
    # link-bound schedule paces itself on the tickets - Eq. 3's max(T_gpu, T_xfer)
    stag = None
    if lay.q_win is not None and lay.logits is not None:
        from paper_2605_17613_amd.runtime import StaggeredLayer
        del dst_k, dst_v
        x = max(2, W // 2)
        link_bw = total / t_swap
        t_gpu = t_draft / n_steps
        kv_req = total / B
        t_xfer = B * kv_req / (x * link_bw)
        t_iter_model = max(t_gpu, t_xfer)
        loop = StaggeredLayer(ctx, lay, 4, host_k, host_v, windows=W, x=x, t_iter=t_iter_model, link_bw=link_bw,
                              hbm_bytes=288e9, model_bytes=0.0, chunk_tokens=chunk_tok)
        loop.run(2 * W)                        # reach the steady state
        torch.cuda.synchronize(); vc.vc_swap_sync(ctx)
        k0, b0, n0 = loop.kicks, loop.bytes_moved, len(loop.log)
        iters = 6 * W
        t0 = time.perf_counter()
        loop.run(iters)
        torch.cuda.synchronize(); vc.vc_swap_sync(ctx)
        t_loop = time.perf_counter() - t0
        wins = [c for (_, _, c) in loop.log[n0:]]
        stag = {"requests": B, "x": x, "windows": W, "iterations": iters, "verifies": len(wins),
                "reloads": loop.kicks - k0, "mean_window": sum(wins) / max(1, len(wins)),
                "ms_per_iteration": t_loop / iters * 1e3, "model_t_gpu_ms": t_gpu * 1e3, "model_t_xfer_ms": t_xfer * 1e3,
                "model_t_iter_ms": t_iter_model * 1e3,
                "link_utilisation": (loop.bytes_moved - b0) / (t_loop * link_bw),
                "tokens_verified_per_s": sum(wins) / t_loop}
        del loop
    return {"bytes": total, "chunks": 2 * len(chunks), "swap_alone_ms": t_swap * 1e3, "swap_GBps": total / t_swap / 1e9,
            "dropped_rows_reload": rows, "staggered_loop": stag,
            "draft_steps": n_steps, "draft_alone_ms": t_draft * 1e3, "both_ms": t_both * 1e3,
            "overlap": (t_draft + t_swap - t_both) / min(t_draft, t_swap), "bytes_ok": ok,
            "model_max_ms": max(t_draft, t_swap) * 1e3, "streamed_verify": streamed}


def measure_small_configs(vc, ctx, torch):
    """Workload configs 0 and 1 as they are.  Config 0 (one sequence of 4096 tokens, 8 q / 2 KV heads,
    int4, window 8, vocab 32000) is pure launch latency: 1.3 MB per draft call.  Config 1 (8 sequences of
    32768 tokens, 2048 kept rows per head, window 16): one draft call moves 68 MB, less than the 256 MB
    last-level cache, so beside the single call on one layer (cache-assisted, said so) the draft is timed
    over 32 distinct layers back to back (34 GB of pools, 2.2 GB gathered per pass)."""
    from tests import synth
    dev = "cuda:0"

    def timed(f, reps, warm):
        for _ in range(warm):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    res = {}
    for idx in (0, 1):
        lay = synth.config(idx, dev)
        nseq, HQ, HKV = len(lay.ctx_len), lay.n_q_heads, lay.n_kv_heads
        N, W = lay.ctx_len[0], lay.win[0]
        if idx == 0:
            kw = dict(blocks=lay.blocks[4], cu_blk=lay.cu_blk[4], max_blk=lay.max_blk[4], bits=4, sum_blk=int(lay.cu_blk[4][-1]))
            dbytes = draft_bytes(nseq, HQ, HKV, blocks=N // 32)
        else:
            kw = dict(pool_k=lay.k_full, pool_v=lay.v_full, cu_ctx=lay.cu_ctx, keep_idx=lay.keep_idx, cu_keep=lay.cu_keep,
                      max_keep=lay.max_keep, sum_keep=int(lay.cu_keep[-1]))
            dbytes = draft_bytes(nseq, HQ, HKV, kept=lay.max_keep)
        out = torch.empty_like(lay.q)
        ws = torch.empty(max(16, vc.vc_draft_workspace_bytes(HQ, HKV, nseq, **kw)), dtype=torch.uint8, device=dev)
        va = dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=N, max_win=W, sum_ctx=N * nseq)
        tw = lay.q_win.shape[0]
        vws = torch.empty(max(16, vc.vc_verify_workspace_bytes(HQ, HKV, nseq, total_win=tw, **va)), dtype=torch.uint8, device=dev)
        vout = torch.empty_like(lay.q_win)
        rows, vocab = lay.logits.shape
        acc = torch.empty(nseq, dtype=torch.int32, device=dev); nxt = torch.empty_like(acc)
        amax = torch.empty(rows, dtype=torch.int32, device=dev)
        aws = torch.empty(max(16, vc.vc_accept_workspace_bytes(rows, vocab)), dtype=torch.uint8, device=dev)
        t_d = timed(lambda: vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV, workspace=ws, **kw), 200, 20)
        t_v = timed(lambda: vc.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, vout, n_seqs=nseq,
                                              workspace=vws, **va), 50, 10)
        t_a = timed(lambda: vc.vc_accept_len(ctx, lay.logits, lay.cu_rows, lay.draft_ids, lay.cu_win, acc, nxt, amax,
                                             workspace=aws), 100, 10)
        vflops = nseq * 4 * HQ * 128 * (W * N + W * (W + 1) / 2)
        vbytes = nseq * (2 * HKV * N * 256 + 2 * HKV * W * 256 + 2 * W * HQ * 256)
        r = {"sequences": nseq, "ctx": N, "window": W,
             "draft_call_us": t_d, "draft_MB": dbytes / 1e6, "draft_GBps_same_layer": dbytes / t_d / 1e3,
             "draft_note": "back-to-back calls on ONE layer: its bytes fit the last-level cache",
             "verify_call_us": t_v, "verify_GBps": vbytes / t_v / 1e3, "verify_TFLOPs": vflops / t_v / 1e6,
             "accept_call_us": t_a, "accept_GBps": rows * vocab * 4 / t_a / 1e3}
        if idx == 1:
            layers = 32
            g = torch.Generator(device=dev); g.manual_seed(synth.SEED_BASE + 100)
            pk = torch.randn((layers,) + tuple(lay.k_full.shape), device=dev, dtype=torch.bfloat16, generator=g)
            pv = torch.randn((layers,) + tuple(lay.v_full.shape), device=dev, dtype=torch.bfloat16, generator=g)
            ql = torch.randn((layers,) + tuple(lay.q.shape), device=dev, generator=g).to(torch.bfloat16)
            ol = torch.empty_like(ql)

            def loop():
                for l in range(layers):
                    kw2 = dict(kw); kw2.update(pool_k=pk[l], pool_v=pv[l])
                    vc.vc_draft_attn(ctx, ql[l], lay.scale, ol[l], n_kv_heads=HKV, workspace=ws, **kw2)

            t_l = timed(loop, 5, 2) / layers
            r.update({"draft_layer_loop_us_per_call": t_l, "draft_layer_loop_GBps": dbytes / t_l / 1e3,
                      "draft_layer_loop_frac_hbm": dbytes / t_l / 1e3 / HBM_PEAK_GBPS, "draft_layer_loop_layers": layers})
            del pk, pv, ql, ol
        res[f"config{idx}"] = r
        del lay, ws, vws
        torch.cuda.empty_cache()
    return res


def measure_config4(vc, ctx, torch, reps=40, warm=25):
    """Workload config 4: 32 sequences of 2048 ... 131072 tokens, each either token-dropped (10 %) or
    int4, verify windows of 4 ... 64 tokens: one draft call, one verify call, one accept call."""
    from tests import synth
    dev = "cuda:0"
    lay = synth.config(4, dev)
    nseq = len(lay.ctx_len)
    HQ, HKV = lay.n_q_heads, lay.n_kv_heads
    kw = dict(pool_k=lay.k_full, pool_v=lay.v_full, cu_ctx=lay.cu_ctx, keep_idx=lay.keep_idx, cu_keep=lay.cu_keep,
              max_keep=lay.max_keep, blocks=lay.blocks[4], cu_blk=lay.cu_blk[4], max_blk=lay.max_blk[4], bits=4,
              sum_keep=int(lay.cu_keep[-1]), sum_blk=int(lay.cu_blk[4][-1]))
    if lay.tail_k is not None:
        kw.update(tail_k=lay.tail_k, tail_v=lay.tail_v, cu_tail=lay.cu_tail, max_tail=lay.max_tail)
    out = torch.empty_like(lay.q)
    ws = torch.empty(max(16, vc.vc_draft_workspace_bytes(HQ, HKV, nseq, **kw)), dtype=torch.uint8, device=dev)
    tw = lay.q_win.shape[0]
    va = dict(k=lay.k_full, v=lay.v_full, cu_ctx=lay.cu_ctx, max_ctx=max(lay.ctx_len), max_win=max(lay.win),
              sum_ctx=sum(lay.ctx_len))
    vws = torch.empty(max(16, vc.vc_verify_workspace_bytes(HQ, HKV, nseq, total_win=tw, **va)), dtype=torch.uint8, device=dev)
    vout = torch.empty_like(lay.q_win)
    rows, vocab = lay.logits.shape
    acc = torch.empty(nseq, dtype=torch.int32, device=dev)
    nxt = torch.empty(nseq, dtype=torch.int32, device=dev)
    amax = torch.empty(rows, dtype=torch.int32, device=dev)
    aws = torch.empty(max(16, vc.vc_accept_workspace_bytes(rows, vocab)), dtype=torch.uint8, device=dev)

    def timed(f):
        for _ in range(warm):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    t_draft = timed(lambda: vc.vc_draft_attn(ctx, lay.q, lay.scale, out, n_kv_heads=HKV, workspace=ws, **kw))
    t_verify = timed(lambda: vc.vc_verify_attn(ctx, lay.q_win, lay.k_win, lay.v_win, lay.cu_win, lay.scale, vout,
                                               n_seqs=nseq, workspace=vws, **va))
    t_accept = timed(lambda: vc.vc_accept_len(ctx, lay.logits, lay.cu_rows, lay.draft_ids, lay.cu_win, acc, nxt, amax,
                                              workspace=aws))
    kept_bytes = int(lay.cu_keep[-1]) * HKV * 512
    rec_bytes = int(lay.cu_blk[4][-1]) * HKV * 5120
    full_bytes = sum(lay.ctx_len) * HKV * 512
    g = HQ // HKV
    flops = sum(4.0 * w * g * 128 * (n + (w + 1) / 2) for n, w in zip(lay.ctx_len, lay.win)) * HKV
    return {"sequences": nseq, "tokens": int(sum(lay.ctx_len)), "int4_sequences": int(sum(1 for b in range(nseq) if int(lay.cu_blk[4][b + 1]) > int(lay.cu_blk[4][b]))),
            "draft_us": t_draft, "draft_GBps": (kept_bytes + rec_bytes) / t_draft / 1e3,
            "verify_us": t_verify, "verify_GBps": full_bytes / t_verify / 1e3, "verify_TFLOPs": flops / t_verify / 1e6,
            "accept_us": t_accept, "accept_GBps": rows * vocab * 4 / t_accept / 1e3}


def measure_round3(vc, ctx, torch, layers=32, N=131072, W=64, vocab=128256, chunk_tok=8192):
    """Workload config 3: one request, `layers` attention layers of the 8B shape at context N.  The
    int4 KV of every layer sits on the GPU, the full bf16 KV in pinned host memory.  One round =
    start the reload of all layers, draft W tokens (W x layers draft calls, the bf16 tail growing),
    verify every layer as its reload lands, accept.  The draft horizon is measured eagerly and as
    one captured HIP graph per step (32 layers x 2 kernels), replayed W times."""
    from tests import synth
    dev = "cuda:0"
    HQ, HKV = 32, 8
    g = torch.Generator(device=dev); g.manual_seed(synth.SEED_BASE + 3)
    row = HKV * 128
    cu_ctx = torch.tensor([0, N], dtype=torch.int32, device=dev)
    nb = N // 32
    cu_blk = torch.tensor([0, nb], dtype=torch.int32, device=dev)
    host_k = torch.empty((layers, N, HKV, 128), dtype=torch.bfloat16, pin_memory=True)
    host_v = torch.empty((layers, N, HKV, 128), dtype=torch.bfloat16, pin_memory=True)
    blocks = torch.empty((layers, HKV * nb, 5120), dtype=torch.uint8, device=dev)
    for l in range(layers):      # full KV made on the GPU, compressed by the library, then moved to the host
        k = torch.randn((N, HKV, 128), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        v = torch.randn((N, HKV, 128), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        vc.vc_compress_quant(ctx, k, v, cu_ctx, cu_blk, 4, nb, blocks[l])
        host_k[l].copy_(k); host_v[l].copy_(v)
    del k, v
    q = torch.randn((layers, 1, HQ, 128), generator=g, device=dev).to(torch.bfloat16)
    q_win = torch.randn((layers, W, HQ, 128), generator=g, device=dev).to(torch.bfloat16)
    k_win = torch.randn((layers, W, HKV, 128), generator=g, device=dev).to(torch.bfloat16)
    v_win = torch.randn((layers, W, HKV, 128), generator=g, device=dev).to(torch.bfloat16)
    logits, ids_star = synth.planted_logits(W, vocab, g)
    prefix = int(torch.randint(0, W + 1, (1,), generator=g, device=dev))
    cu_win = torch.tensor([0, W], dtype=torch.int32, device=dev)
    draft_ids = synth.drafts_with_prefix(ids_star.clone(), [0, W], [prefix], vocab).to(torch.int32).contiguous()
    stage_k = torch.empty((layers, N, HKV, 128), dtype=torch.bfloat16, device=dev)
    stage_v = torch.empty_like(stage_k)
    scale = 1.0 / math.sqrt(128)
    out = torch.empty((layers, 1, HQ, 128), dtype=torch.bfloat16, device=dev)
    vout = torch.empty_like(q_win)
    cu_tail = torch.zeros(2, dtype=torch.int32, device=dev)
    cu_tail_steps = [torch.tensor([0, s], dtype=torch.int32, device=dev) for s in range(W)]
    dkw = lambda l: dict(blocks=blocks[l], cu_blk=cu_blk, max_blk=nb, bits=4, sum_blk=nb, tail_k=k_win[l], tail_v=v_win[l],
                         cu_tail=cu_tail, max_tail=W - 1)
    vkw = lambda l: dict(k=stage_k[l], v=stage_v[l], cu_ctx=cu_ctx, max_ctx=N, max_win=W, sum_ctx=N)
    ws = torch.empty(max(vc.vc_draft_workspace_bytes(HQ, HKV, 1, **dkw(0)),
                         vc.vc_verify_workspace_bytes(HQ, HKV, 1, total_win=W, **vkw(0))), dtype=torch.uint8, device=dev)
    acc = torch.empty(1, dtype=torch.int32, device=dev); nxt = torch.empty_like(acc)
    amax = torch.empty(W, dtype=torch.int32, device=dev)
    aws = torch.empty(vc.vc_accept_workspace_bytes(W, vocab), dtype=torch.uint8, device=dev)
    layer_bytes = N * row * 2
    chunks = [(t * row * 2, t * row * 2, min(chunk_tok, N - t) * row * 2) for t in range(0, N, chunk_tok)]

    def draft_step():
        for l in range(layers):
            vc.vc_draft_attn(ctx, q[l], scale, out[l], n_kv_heads=HKV, workspace=ws, **dkw(l))

    def horizon_eager():
        for s in range(W):
            cu_tail.copy_(cu_tail_steps[s])
            draft_step()

    def swap_all():
        last = []
        for l in range(layers):
            vc.vc_swap_in(ctx, host_k[l], stage_k[l], chunks)
            last.append(vc.vc_swap_in(ctx, host_v[l], stage_v[l], chunks) + len(chunks) - 1)
        return last

    def verify_all(last):
        for l in range(layers):
            if last is not None:
                vc.vc_swap_wait(ctx, last[l])
            vc.vc_verify_attn(ctx, q_win[l], k_win[l], v_win[l], cu_win, scale, vout[l], n_seqs=1, workspace=ws, **vkw(l))
        vc.vc_accept_len(ctx, logits, cu_win, draft_ids, cu_win, acc, nxt, amax, workspace=aws)

    def wall(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter(); r = fn(); torch.cuda.synchronize(); vc.vc_swap_sync(ctx)
        return time.perf_counter() - t0, r

    draft_step(); torch.cuda.synchronize()
    t_eager, _ = wall(horizon_eager)
    # one draft step (all layers) as a HIP graph; the tail length lives in device memory, so the
    # same graph serves every step of the horizon
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        draft_step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            draft_step()
    torch.cuda.synchronize()

    def horizon_graph():
        for s in range(W):
            cu_tail.copy_(cu_tail_steps[s])
            graph.replay()

    ref = None
    cu_tail.copy_(cu_tail_steps[W - 1]); draft_step(); torch.cuda.synchronize(); ref = out.clone()
    t_graph, _ = wall(horizon_graph)
    graph_same = bool(torch.equal(ref.view(torch.int16), out.view(torch.int16)))
    t_swap, last = wall(swap_all)
    t_verify, _ = wall(lambda: verify_all(None))

    def round_():
        last = swap_all()
        horizon_graph()
        verify_all(last)

    t_round, _ = wall(round_)
    a = int(acc)
    draft_bytes = sum(layers * (HKV * nb * 5120 + s * HKV * 512 + 2 * HQ * 256) for s in range(W))
    return {"layers": layers, "ctx": N, "window": W, "int4_GB": blocks.numel() / 1e9, "full_kv_GB": 2 * layers * layer_bytes / 1e9,
            "draft_horizon_eager_ms": t_eager * 1e3, "draft_horizon_graph_ms": t_graph * 1e3, "graph_equals_eager": graph_same,
            "draft_GBps_graph": draft_bytes / t_graph / 1e9, "ms_per_drafted_token": t_graph / W * 1e3,
            "swap_alone_ms": t_swap * 1e3, "swap_GBps": 2 * layers * layer_bytes / t_swap / 1e9,
            "verify_accept_ms": t_verify * 1e3, "round_ms": t_round * 1e3,
            "model_max_ms": max(t_graph, t_swap) * 1e3 + t_verify / layers * 1e3,
            "accept_len": a, "planted_prefix": prefix, "accept_exact": a == prefix,
            "tokens_per_round": a + 1, "tokens_per_s": (a + 1) / t_round}


def cpu_baseline(lay, torch, np, HQ, HKV, N):
    """The fp64 oracle, as it stands, on all host cores of the box: int4 draft attention (all g query
    heads) of a bounded sample of (sequence, KV head) pairs at full context, one pair per task, in
    worker processes (the oracle is single-threaded numpy).  Rate = record bytes / wall time."""
    from tests import oracle_pool as P
    blocks = lay.blocks[4]
    nb = N // 32
    cu = np.array([0, nb], dtype=np.int32)
    g = HQ // HKV
    workers = P.n_workers()
    nseq = lay.q.shape[0]
    all_pairs = [(b, kvh) for b in range(nseq) for kvh in range(HKV)]
    pairs = all_pairs[:min(len(all_pairs), 8 * workers)]             # about 10 - 20 s of wall time
    tasks = []
    for (b, kvh) in pairs:
        start = int(lay.cu_blk[4][b]) * HKV + kvh * nb
        tasks.append({"q": lay.q[b, kvh * g:(kvh + 1) * g].contiguous().view(torch.int16).cpu().numpy().view(np.uint16),
                      "scale": lay.scale,
                      "kv": dict(blocks=blocks[start:start + nb].cpu().numpy(), cu_blk=cu, bits=4)})
    try:
        P.run(P.draft_task, tasks[:workers])                          # start the workers (imports) outside the timed part
        t0 = time.perf_counter()
        res = P.run(P.draft_task, tasks)
        wall = time.perf_counter() - t0
    finally:
        P.shutdown()
    nbytes = len(pairs) * nb * 5120
    in_oracle = sum(r[1] for r in res)
    return {"value": nbytes / wall / 1e9, "unit": "GB/s", "cores": workers, "kind": "oracle",
            "sample": f"int4 draft attention of {len(pairs)} of {len(all_pairs)} (sequence, KV head) pairs at ctx {N}, all {g} query heads each "
                      f"({nbytes / 1e6:.1f} MB of records; {wall:.1f} s wall on {workers} worker processes, {in_oracle:.1f} s summed inside the oracle)"}


if __name__ == "__main__":
    main()
