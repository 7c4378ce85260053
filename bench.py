#!/usr/bin/env python3
"""Benchmark of the filtered-attention hot path on one MI355X.

One step = one pass of the whole path (score -> fuse -> select -> compact -> attend) over one
batch of seeded synthetic Q/K/V, through the C ABI, inputs resident in HBM.  The default
workload is the LLaMA-2-7B-shaped layer (bf16, batch 8, 32 heads x 128, seq 4096) at pruning
ratio 0.5, the configuration the headline metric is quoted on.

Prints ONE JSON line.  Besides the whole-path throughput it carries
  roofline      the dominant kernel (bf16 MFMA attention over the kept tokens): useful flops
                2 d m (m + 1) Hq B per launch / its average duration measured with events on
                the launch stream inside the timed steps, against the 2.5 PFLOP/s dense bf16
                peak;
  cpu_baseline  the CPU oracle, as it stands, timed on the host cores over a bounded sample
                (whole path on the batch rows of the same workload; one row when n > 4096);
  ceilings      what this device reaches on a plain streaming read of the K tensor and on
                back-to-back bf16 MFMAs (the library's probes), next to the vendor peaks;
  other_ratios  the same workload at the other pruning ratio its configuration names (0.25),
                timed the same way (context: `value` is the 50 % line).
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

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
METRIC = "filtered-attention tokens/s (score+compact+attend) @50% prune"


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel, from the committed counter summary."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", type=int, default=1, help="index into the workload table")
    ap.add_argument("--ratio", type=float, default=0.5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prewarm-seconds", type=float, default=0.25,
                    help="untimed steps run for this long before the W warm-up steps, to bring "
                         "the device out of its idle clocks (0 for counter-collection runs)")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the probes and the other pruning ratios (for profiler runs: only "
                         "the headline configuration's kernels are launched)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of known size (to scale HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this path runs on one GPU; rows of a batch are independent, so "
                 "more GPUs would just take disjoint batch rows. Run with --gpus 1.")

    import numpy as np
    import torch

    from paper_2512_07090_amd import binding as B
    from paper_2512_07090_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.copy_calibration:
        # a plain elementwise copy kernel: reads and writes exactly `nbytes` each
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": nbytes, "copy_bytes_written": nbytes, "copies": 3}))
        return
    B.lib()  # fail loudly if the HIP library is not built

    w = synth.workload(args.workload)
    q, k, v, _ = synth.make_qkv(w)
    dev = "cuda:0"
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    p = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, args.ratio)
    buf = B.Buffers(p, dev)
    ctx = B.Context(0)
    m = buf.m
    K = min(args.steps, 256)

    def step():
        ctx.tf_filtered_attention(p, qd, kd, vd, buf.keep, buf.kept_idx, buf.fused, buf.tau,
                                  buf.O, buf.ws)

    # Bring the device to its working state first: the first tens of milliseconds after idle
    # run 15-20 % slower (clocks ramping up), whatever W is.  Not timed.
    t_pre = time.perf_counter()
    while time.perf_counter() - t_pre < args.prewarm_seconds:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly K steps, events on the launch stream plus a host clock
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(K):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / K
    ms_per_step = e0.elapsed_time(e1) / K
    tokens = w.batch * w.seq
    value = tokens / (ms_per_step * 1e-3)

    # the same K steps again with the library's per-stage events on the launch stream
    ctx.tf_stage_timing_enable(True)
    for _ in range(K):
        step()
    stage_ms, n_calls = ctx.tf_stage_timing_read()
    ctx.tf_stage_timing_enable(False)
    stage_ms = [x / max(n_calls, 1) for x in stage_ms]
    stages = dict(zip(B.STAGE_NAMES, stage_ms))

    attn_flops = 2.0 * w.head_dim * m * (m + 1) * w.n_q_heads * w.batch
    attn_tflops = attn_flops / (stages["attend"] * 1e-3) / 1e12
    esize = 4 if w.dtype == "f32" else 2
    score_bytes = 2.0 * w.batch * w.n_kv_heads * w.seq * w.head_dim * esize
    score_gbs = score_bytes / (stages["score"] * 1e-3) / 1e9
    roofline = {"kernel": "attend_bf16_kernel" if w.dtype == "bf16" else "attend_f32_kernel",
                "bound": "mfma", "achieved": round(attn_tflops, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                "traffic": read_traffic("attend_bf16_%s_pmc.txt" % w.name),
                "avg_kernel_ms": round(stages["attend"], 4)}
    score_roofline = {"kernel": "scan_score_kernel", "bound": "hbm",
                      "achieved": round(score_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                      "frac": round(score_gbs / PEAK_HBM_GBS, 4),
                      "traffic": read_traffic("scan_score_%s_pmc.txt" % w.name),
                      "avg_kernel_ms": round(stages["score"], 4)}

    # on-box ceilings (measured after the timed region)
    ceilings = None
    if not args.headline_only:
        ceilings = {"hbm_read_GBps": round(ctx.tf_probe_hbm_read(kd), 1),
                    "mfma_bf16_TFLOPs": round(ctx.tf_probe_mfma_bf16(20000), 1),
                    "vendor_hbm_GBps": PEAK_HBM_GBS, "vendor_mfma_bf16_TFLOPs": PEAK_BF16_TFLOPS}

    # the workload's other pruning ratios, timed like the headline
    other = {}
    for r2 in w.prune_ratios:
        if abs(r2 - args.ratio) < 1e-12 or args.headline_only:
            continue
        p2 = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, r2)
        b2 = B.Buffers(p2, dev)

        def step2():
            ctx.tf_filtered_attention(p2, qd, kd, vd, b2.keep, b2.kept_idx, b2.fused, b2.tau,
                                      b2.O, b2.ws)
        for _ in range(args.warmup):
            step2()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(K):
            step2()
        e1.record()
        torch.cuda.synchronize()
        ms2 = e0.elapsed_time(e1) / K
        fl2 = 2.0 * w.head_dim * b2.m * (b2.m + 1) * w.n_q_heads * w.batch
        other["%g" % r2] = {"ms_per_step": round(ms2, 4), "tokens_per_s": round(tokens / (ms2 * 1e-3), 1),
                            "kept_per_row": b2.m, "attn_flops_per_step": fl2}
        del b2

    # scoring-stage variants on the same tensors: the incremental anchor of Eq. 1 and the
    # single-tensor scores of Table 7 (each timed like the headline, whole path)
    variants = {}
    if not args.headline_only:
        for name, kw in (("ema_gamma_0.9", dict(ema_gamma=0.9)),
                         ("key_only", dict(fusion=B.TF_FUSE_KEY_ONLY))):
            p3 = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, args.ratio, **kw)
            b3 = B.Buffers(p3, dev)

            def step3():
                ctx.tf_filtered_attention(p3, qd, kd, vd, b3.keep, b3.kept_idx, b3.fused,
                                          b3.tau, b3.O, b3.ws)
            for _ in range(args.warmup):
                step3()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(K):
                step3()
            e1.record()
            torch.cuda.synchronize()
            ms3 = e0.elapsed_time(e1) / K
            ctx.tf_stage_timing_enable(True)
            for _ in range(K):
                step3()
            st3, n3 = ctx.tf_stage_timing_read()
            ctx.tf_stage_timing_enable(False)
            variants[name] = {"ms_per_step": round(ms3, 4), "score_ms": round(st3[0] / max(n3, 1), 4),
                              "attend_ms": round(st3[5] / max(n3, 1), 4)}
            del b3

        # the online decision (adaptive threshold of Eq. 4) in place of the exact count: whole
        # path, and the decision kernel alone on the scores of the headline run
        p4 = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, args.ratio, warmup=8)
        b4 = B.Buffers(p4, dev)
        idx4 = torch.empty((w.batch, w.seq), dtype=torch.int32, device=dev)
        cnt4 = torch.empty((w.batch,), dtype=torch.int32, device=dev)

        def step4():
            ctx.tf_filtered_attention_online(p4, 0.02, 0.5, qd, kd, vd, b4.keep, idx4, cnt4,
                                             b4.fused, b4.tau, b4.O, b4.ws)

        def sel4():
            ctx.tf_select_online(p4, 0.02, 0.5, buf.fused, b4.keep, idx4, cnt4, b4.tau, b4.ws)
        res4 = []
        for fn in (step4, sel4):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(K):
                fn()
            e1.record()
            torch.cuda.synchronize()
            res4.append(e0.elapsed_time(e1) / K)
        variants["online_eta_0.02"] = {"ms_per_step": round(res4[0], 4), "select_online_ms": round(res4[1], 4),
                                       "kept_per_row": [int(x) for x in cnt4.cpu().tolist()]}
        del b4

        # the per-token form: the workload's tokens one at a time (fills the anchors, the
        # controller state and the cache of kept tokens), then K more steps timed; the
        # attention of a step streams the row's cache once (HBM-bound)
        p5 = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, args.ratio, warmup=8)
        b5 = B.DecodeBuffers(p5, w.seq + K + args.warmup, dev)
        qs = qd.permute(2, 0, 1, 3).contiguous()
        ks = kd.permute(2, 0, 1, 3).contiguous()
        vs = vd.permute(2, 0, 1, 3).contiguous()
        ctx.tf_decode_init(p5, b5.state, 0.5)

        def step5(t):
            t %= w.seq
            ctx.tf_decode_step(p5, 0.02, b5.state, qs[t], ks[t], vs[t], b5.o, b5.skip, b5.fused, b5.ws)
        for t in range(w.seq + args.warmup):
            step5(t)
        len0 = b5.cache_len.sum().item()
        torch.cuda.synchronize()
        e0.record()
        for t in range(K):
            step5(w.seq + args.warmup + t)
        e1.record()
        torch.cuda.synchronize()
        ms5 = e0.elapsed_time(e1) / K
        len1 = b5.cache_len.sum().item()
        kept5 = (len1 - len0) / (K * w.batch)               # fraction of the timed tokens that attended
        esz = 2 if w.dtype == "bf16" else 4
        cache_bytes = 0.5 * (len0 + len1) * kept5 * w.n_kv_heads * w.head_dim * 2 * esz
        variants["decode_step"] = {"ms_per_step": round(ms5, 4),
                                   "tokens_per_s": round(w.batch / (ms5 * 1e-3), 1),
                                   "cache_rows_per_batch_row": round(0.5 * (len0 + len1) / w.batch, 1),
                                   "kept_fraction": round(kept5, 3),
                                   "cache_GBps": round(cache_bytes / (ms5 * 1e-3) / 1e9, 1)}
        del b5, qs, ks, vs

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: the whole path on the same tensors; every batch row of the default
        # workload (a few seconds on 16 cores), one row of the long-context ones, whose
        # quadratic attention would take minutes
        rows = w.batch if w.seq <= 4096 else 1
        qs, ks, vs = q[:rows], k[:rows], v[:rows]
        t0 = time.perf_counter()
        ref = oracle.filtered_attention(qs, ks, vs, args.ratio)
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": round(rows * w.seq / dt, 1), "unit": "tokens/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": "whole path on batch rows 0..%d of %d (%d tokens), %.1f s" %
                                  (rows - 1, w.batch, rows * w.seq, dt)}
        # while the reference is at hand: the benchmarked outputs agree with it
        fused = buf.fused[0].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(fused - ref["fused"][0]) <= 1e-5 * np.abs(ref["fused"][0]) + 1e-6)

    out = {"metric": METRIC if abs(args.ratio - 0.5) < 1e-12 else
           METRIC.replace("@50%", "@%g%%" % (100 * args.ratio)),
           "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": w.dtype, "data": "synthetic",
           "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads,
                      "n_kv_heads": w.n_kv_heads, "seq": w.seq, "head_dim": w.head_dim,
                      "prune_ratio": args.ratio, "kept_per_row": m},
           "roofline": roofline, "cpu_baseline": cpu_baseline,
           "stages_ms": {k_: round(v_, 4) for k_, v_ in stages.items()},
           "score_roofline": score_roofline, "ceilings": ceilings, "other_ratios": other,
           "score_variants": variants,
           "host_ms_per_step": round(wall_ms, 4)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
