#!/usr/bin/env python3
"""Benchmark of the filtered-attention hot path on one MI355X.

One step = one pass of the whole path (score -> fuse -> select -> compact -> attend) over one
batch of seeded synthetic Q/K/V, through the C ABI, inputs resident in HBM.  The headline
workload is the LLaMA-2-7B-shaped layer (bf16, batch 8, 32 heads x 128, seq 4096) at pruning
ratio 0.5, the configuration the metric is quoted on.

Prints ONE JSON line.  Besides the whole-path throughput it carries
  roofline      the dominant kernel (bf16 MFMA attention over the kept tokens): useful flops
                2 d m (m + 1) Hq B per launch / its average duration measured with events on
                the launch stream inside the timed steps, against the 2.5 PFLOP/s dense bf16
                peak; `traffic` is the HBM byte count of one launch taken from the committed
                rocprofv3 counter summary (a separate profiler run of this command, not
                measured in this run; `traffic_source` names the file);
  cpu_baseline  the CPU oracle, as it stands, timed on the host cores over a bounded sample of
                the headline workload; the same call checks the benchmarked scores, decisions
                and every attention output row of the sample;
  per_workload  all five workloads of the benchmark definition, each timed the same way
                (mean and median step, per-stage times, scoring GB/s and attention TFLOP/s as
                fractions of the vendor peaks) with the oracle timed beside each on a bounded
                sample (plus the one-thread oracle time on the smallest workload);
  ceilings      what this device reaches on a plain streaming read of the K tensor and on
                back-to-back bf16 MFMAs (the library's probes), next to the vendor peaks;
  other_ratios  the headline workload at the other pruning ratio its configuration names;
  score_variants  the rows built beyond the headline path, on the headline workload.

Stage times come from events the library records between its launches (a second pass of K
steps); "select_compact" is the decision and compaction launch, "attend" includes the launch
that zero-fills filtered rows on the fp32 path.  Every stage figure carries the cost of one
event record (a few microseconds).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
METRIC = "filtered-attention tokens/s (score+compact+attend) @50% prune"


def read_traffic(name):
    """HBM bytes per launch of a kernel, from the committed counter summary (or None)."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1].split()[0]), "profiles/" + name
    except OSError:
        pass
    return None, None


def host_cores():
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


class Timed:
    """One workload resident on the device plus the three timing passes over it."""

    def __init__(self, B, synth, ctx, w, ratio, dev="cuda:0", **param_kw):
        import torch
        self.torch, self.B, self.ctx, self.w, self.ratio = torch, B, ctx, w, ratio
        self.q, self.k, self.v, _ = synth.make_qkv(w)
        self.qd, self.kd, self.vd = self.q.to(dev), self.k.to(dev), self.v.to(dev)
        self.p = B.make_params(tuple(self.q.shape), tuple(self.k.shape), self.q.dtype, ratio, **param_kw)
        self.buf = B.Buffers(self.p, dev)
        self.m = self.buf.m

    def step(self):
        b = self.buf
        self.ctx.tf_filtered_attention(self.p, self.qd, self.kd, self.vd, b.keep, b.kept_idx,
                                       b.fused, b.tau, b.O, b.ws)

    def run(self, K, W, prewarm_s):
        """-> dict: mean ms per step over exactly K steps in one bracket, the median of K
        individually bracketed steps, per-stage means."""
        torch, B = self.torch, self.B
        # Bring the device to its working state first: the first tens of milliseconds after
        # idle run 15-20 % slower (clocks ramping up), whatever W is.  Not timed.
        t_pre = time.perf_counter()
        while time.perf_counter() - t_pre < prewarm_s:
            for _ in range(10):
                self.step()
            torch.cuda.synchronize()
        for _ in range(W):
            self.step()
        torch.cuda.synchronize()
        # timed region: exactly K steps, events on the launch stream plus a host clock
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(K):
            self.step()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / K
        mean_ms = e0.elapsed_time(e1) / K
        # the same K steps, each between its own pair of events: the median step
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        ev[0].record()
        for i in range(K):
            self.step()
            ev[i + 1].record()
        torch.cuda.synchronize()
        each = [ev[i].elapsed_time(ev[i + 1]) for i in range(K)]
        # and once more with the library's per-stage events on the launch stream
        self.ctx.tf_stage_timing_enable(True)
        for _ in range(K):
            self.step()
        st, n_calls = self.ctx.tf_stage_timing_read()
        self.ctx.tf_stage_timing_enable(False)
        st = dict(zip(B.STAGE_NAMES, [x / max(n_calls, 1) for x in st]))
        stages = {"score": st["score"], "fuse": st["fuse"],
                  "select_compact": st["select"] + st["compact"],
                  "attend": st["zero_rows"] + st["attend"]}
        return {"ms_per_step": mean_ms, "ms_per_step_median": statistics.median(each),
                "median_over": K, "host_ms_per_step": wall_ms, "stages_ms": stages}

    def rooflines(self, stages):
        w, m = self.w, self.m
        esize = 4 if w.dtype == "f32" else 2
        n_tensors = 1 if self.p.fusion in (self.B.TF_FUSE_KEY_ONLY, self.B.TF_FUSE_VALUE_ONLY) else 2
        score_bytes = float(n_tensors) * w.batch * w.n_kv_heads * w.seq * w.head_dim * esize
        score_gbs = score_bytes / (stages["score"] * 1e-3) / 1e9
        attn_flops = 2.0 * w.head_dim * m * (m + 1) * w.n_q_heads * w.batch
        attn_tflops = attn_flops / (stages["attend"] * 1e-3) / 1e12
        return score_bytes, score_gbs, attn_flops, attn_tflops

    def oracle_baseline(self, rows, prefix=None, threads_note=None):
        """The oracle's whole path on `rows` batch rows (optionally on the first `prefix`
        tokens only), timed; the benchmarked outputs are checked against it while it is at hand.
        -> cpu_baseline dict."""
        import numpy as np
        import oracle
        w = self.w
        n = prefix or w.seq
        qs, ks, vs = (x[:rows, :, :n] for x in (self.q, self.k, self.v))
        t0 = time.perf_counter()
        ref = oracle.filtered_attention(qs, ks, vs, self.ratio, with_attention=False)
        t_score = time.perf_counter() - t0
        fused = self.buf.fused[:rows, :n].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(fused - ref["fused"]) <= 1e-5 * np.abs(ref["fused"]) + 1e-6), \
            "benchmarked scores differ from the oracle's"
        checked = "scores"
        if prefix is None:
            # the oracle's attention on the kept set the device chose (equal to the oracle's
            # own outside the 1e-5 band around the threshold, which is asserted)
            keep_g = self.buf.keep[:rows].cpu().numpy()
            idx_g = self.buf.kept_idx[:rows].cpu().numpy()
            s32 = ref["fused"].astype(np.float32).astype(np.float64)
            for b in range(rows):
                diff = np.nonzero(keep_g[b] != ref["keep"][b])[0]
                assert np.all(np.abs(s32[b][diff] - float(ref["tau"][b])) <= 1e-5), \
                    "benchmarked mask differs from the oracle's outside the threshold band"
            t1 = time.perf_counter()
            O_ref = oracle.attend(qs, ks, vs, idx_g)
            t_att = time.perf_counter() - t1
            tol = 1e-4 if w.dtype == "f32" else 2e-2
            for b in range(rows):
                O_g = self.buf.O[b].float().cpu().numpy().astype(np.float64)
                err = np.abs(O_g - O_ref[b]).max()
                assert err <= tol, "benchmarked attention output differs: max-abs %.3e" % err
            checked = "scores, mask and every attention output row"
        else:
            # a prefix of the row: scores are causal, so they are the device's; the decision over
            # a prefix is another problem than the one over the whole row, so it is only timed
            t1 = time.perf_counter()
            oracle.attend(qs, ks, vs, ref["kept_idx"])
            t_att = time.perf_counter() - t1
        dt = t_score + t_att
        cores = min(oracle.num_threads(), host_cores())
        what = ("batch rows 0..%d of %d" % (rows - 1, w.batch)) + \
               ("" if prefix is None else ", first %d of %d tokens" % (n, w.seq))
        return {"value": round(rows * n / dt, 1), "unit": "tokens/s", "cores": cores,
                "omp_max_threads": oracle.num_threads(), "affinity_cores": host_cores(),
                "kind": "oracle",
                "sample": "whole path on %s (%d tokens), %.1f s; checked against it: %s" %
                          (what, rows * n, dt, checked)}


def baseline_sample(w):
    """(rows, prefix) of the bounded oracle sample for a workload: all rows of the 4096-token
    workloads, one row of the 8192-token one, the first 16384 tokens of the 32768-token one
    (its quadratic attention would take most of a minute)."""
    if w.seq <= 4096:
        return w.batch, None
    if w.seq <= 8192:
        return 1, None
    return 1, 16384


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", type=int, default=1, help="index of the headline workload")
    ap.add_argument("--ratio", type=float, default=0.5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prewarm-seconds", type=float, default=0.25,
                    help="untimed steps run for this long before the W warm-up steps, to bring "
                         "the device out of its idle clocks (0 for counter-collection runs)")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the headline configuration's kernels are launched (for profiler "
                         "runs): no probes, other ratios, variants or other workloads")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of known size (to scale HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this path runs on one GPU; rows of a batch are independent, so "
                 "more GPUs would just take disjoint batch rows. Run with --gpus 1.")

    import numpy as np  # noqa: F401
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

    dev = "cuda:0"
    ctx = B.Context(0)
    K = min(args.steps, 256)
    w = synth.workload(args.workload)
    head = Timed(B, synth, ctx, w, args.ratio)
    res = head.run(K, args.warmup, args.prewarm_seconds)
    stages = res["stages_ms"]
    ms_per_step = res["ms_per_step"]
    tokens = w.batch * w.seq
    value = tokens / (ms_per_step * 1e-3)
    m = head.m
    q, k = head.q, head.k
    qd, kd, vd, buf = head.qd, head.kd, head.vd, head.buf

    score_bytes, score_gbs, attn_flops, attn_tflops = head.rooflines(stages)
    kname = "attend_bf16_kernel" if w.dtype == "bf16" else "attend_f32_kernel"
    tr_a, src_a = read_traffic("attend_bf16_%s_pmc.txt" % w.name)
    tr_s, src_s = read_traffic("scan_score_%s_pmc.txt" % w.name)
    roofline = {"kernel": kname, "bound": "mfma", "achieved": round(attn_tflops, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4), "traffic": tr_a,
                "traffic_source": src_a and src_a + " (rocprofv3 --pmc run, not this run)",
                "avg_kernel_ms": round(stages["attend"], 4)}
    score_roofline = {"kernel": "scan_score_kernel", "bound": "hbm",
                      "achieved": round(score_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                      "frac": round(score_gbs / PEAK_HBM_GBS, 4), "traffic": tr_s,
                      "traffic_source": src_s and src_s + " (rocprofv3 --pmc run, not this run)",
                      "avg_kernel_ms": round(stages["score"], 4)}

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

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
        head.step()                      # the headline outputs (the variants reused nothing of buf)
        torch.cuda.synchronize()
        rows, prefix = baseline_sample(w)
        cpu_baseline = head.oracle_baseline(rows, prefix)

    def summary(t, r):
        sb, sg, af, at = t.rooflines(r["stages_ms"])
        ww = t.w
        d = {"ratio": t.ratio, "kept_per_row": t.m, "steps": r["median_over"],
             "ms_per_step": round(r["ms_per_step"], 4),
             "ms_per_step_median": round(r["ms_per_step_median"], 4),
             "tokens_per_s": round(ww.batch * ww.seq / (r["ms_per_step"] * 1e-3), 1),
             "stages_ms": {k_: round(v_, 4) for k_, v_ in r["stages_ms"].items()},
             "score": {"algorithmic_bytes": sb, "GBps": round(sg, 1), "frac_of_hbm_peak": round(sg / PEAK_HBM_GBS, 4)},
             "attend": {"algorithmic_flops": af, "TFLOPs": round(at, 2),
                        "frac_of_bf16_mfma_peak": round(at / PEAK_BF16_TFLOPS, 4) if ww.dtype == "bf16" else None,
                        "note": None if ww.dtype == "bf16" else "fp32 correctness path: plain FMA, no MFMA peak applies"}}
        return d

    # every workload of the benchmark definition, timed like the headline
    per_workload = {}
    if not args.headline_only:
        per_workload[w.name] = summary(head, res)
        per_workload[w.name]["cpu_baseline"] = cpu_baseline
        del head, buf, qd, kd, vd
        torch.cuda.empty_cache()
        for i in range(len(synth.WORKLOADS)):
            wi = synth.workload(i)
            if wi.name == w.name:
                continue
            t = Timed(B, synth, ctx, wi, 0.5)
            Ki = max(20, min(K, 100))
            ri = t.run(Ki, min(args.warmup, 20), 0.1)
            per_workload[wi.name] = summary(t, ri)
            if not args.no_cpu_baseline:
                rows, prefix = baseline_sample(wi)
                cb = t.oracle_baseline(rows, prefix)
                if i == 0:
                    # the smallest workload once more on one thread
                    import oracle
                    env_threads = oracle.num_threads()
                    oracle.set_num_threads(1)
                    t1 = time.perf_counter()
                    oracle.filtered_attention(t.q, t.k, t.v, 0.5)
                    cb["one_thread_tokens_per_s"] = round(wi.batch * wi.seq / (time.perf_counter() - t1), 1)
                    oracle.set_num_threads(env_threads)
                per_workload[wi.name]["cpu_baseline"] = cb
            del t
            torch.cuda.empty_cache()
        per_workload = dict(sorted(per_workload.items()))

    out = {"metric": METRIC if abs(args.ratio - 0.5) < 1e-12 else
           METRIC.replace("@50%", "@%g%%" % (100 * args.ratio)),
           "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "ms_per_step_median": round(res["ms_per_step_median"], 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": w.dtype, "data": "synthetic",
           "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads,
                      "n_kv_heads": w.n_kv_heads, "seq": w.seq, "head_dim": w.head_dim,
                      "prune_ratio": args.ratio, "kept_per_row": m},
           "roofline": roofline, "cpu_baseline": cpu_baseline,
           "stages_ms": {k_: round(v_, 4) for k_, v_ in stages.items()},
           "score_roofline": score_roofline, "ceilings": ceilings, "other_ratios": other,
           "score_variants": variants, "per_workload": per_workload,
           "host_ms_per_step": round(res["host_ms_per_step"], 4)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
