#!/usr/bin/env python3
"""Benchmark of the speculative-decoding hot path on one MI355X.

A step is one whole speculative decode of the batch: reset to the post-prefill state, then
rounds (draft proposal, single-pass verification, acceptance/commit/rollback) until every series
has its horizon.  Inputs (weights, KV cache of the context) are resident in HBM before the
timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg2] [--sigma 1.0]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--sigma", type=float, default=None)
    ap.add_argument("--batch", type=int, default=None, help="series in the batch (default: the configuration's; other sizes are side experiments)")
    ap.add_argument("--sample-proposals", action="store_true", help="ablation: x_i = mu_q + sigma_q eps")
    ap.add_argument("--fallback-r", type=float, default=0.0, help="ablation: fallback / bonus noise scale")
    ap.add_argument("--naive-verify", action="store_true", help="ablation: one target pass per prefix")
    ap.add_argument("--threshold-rule", action="store_true", help="variant: accept iff ||x - mu_p||_d^2 <= sigma^2")
    ap.add_argument("--batch-sync", action="store_true", help="variant: all series keep the batch's smallest accepted count")
    ap.add_argument("--fused-draft", choices=["auto", "on", "off"], default="auto",
                    help="the draft phase as one launch: where the library picks it (auto), wherever supported (on), never (off)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-series", type=int, default=128, help="series in the oracle's bounded sample (~15 s of CPU work at cfg2)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB copy kernel 5 times (known traffic, to scale profiler memory counters)")
    return ap.parse_args()


def decode_spec(sess):
    sess.reset_decode()
    return sess.run_rounds()[0]   # rounds until every series has its horizon (the loop lives in the library)


def decode_target_only(sess, T):
    sess.reset_decode()
    for _ in range(T):
        sess.target_step()


def timed(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()       # waits for every stream of the device, the session's included
    return (time.perf_counter() - t0) / steps


def phase_times(torch, sess, reps=20):
    """hipEvent time of one draft proposal, one verification, one acceptance, one target-only
    step (each repeated from the post-prefill state)."""
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {}
    for name, fn in (("draft", sess.draft_propose), ("verify", sess.target_verify),
                     ("accept", sess.accept_commit), ("target_step", sess.target_step)):
        tot = 0.0
        for _ in range(reps):
            sess.reset_decode()
            if name == "accept":
                sess.draft_propose(); sess.target_verify()
            a, b = ev(), ev()
            a.record(sess.stream); fn(); b.record(sess.stream)   # events on the stream the kernels run on
            torch.cuda.synchronize()
            tot += a.elapsed_time(b)
        out[name] = tot / reps
    return out


# HBM bytes per launch of each kernel family from rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by the
# copy-kernel calibration (profiles/traffic_cfg2_bench.md has the commands, raw values and factors)
TRAFFIC = {"cfg2": {"resid": 12815008, "qkv": 8749837, "gelu": 9236849, "attn": 13896280, "head": 2648011,
                    "embed": 3006556, "accept": 818654, "draft": 113752075}}
PEAK = {"bf16": 2500.0, "fp32": 157.3}   # dense MFMA bf16 / vector fp32, TFLOP/s
HBM_PEAK = 8000.0                        # GB/s


def kernel_rooflines(sess, dtype, steps, workload, cfg=None):
    """Per kernel family: HIP-event time of every launch during `steps` speculative decodes
    (kernel-by-kernel launches on the session's stream), and the algorithmic work they did."""
    from paper_2511_18191_amd.binding import KERNEL_CLASSES
    out = {}
    for cls, name in enumerate(KERNEL_CLASSES):
        sess.profile_begin(cls)
        for _ in range(steps):
            decode_spec(sess)
        n, ms, work = sess.profile_end()
        if n == 0:
            continue
        if name == "draft":
            # one launch runs all K draft steps; every workgroup streams the draft's weights once per step
            # through its compute unit's vector-memory path (64 B/clk at 2.4 GHz = 153.6 GB/s per unit)
            out[name] = dict(bound="cu_stream", launches=n, avg_us=ms * 1e3 / n, total_ms=ms,
                             mfma_tflops=work / (ms * 1e-3) / 1e12, peak_gbs_per_cu=153.6, unit="GB/s per CU",
                             traffic=TRAFFIC.get(workload, {}).get(name))
            if cfg is not None:
                d = cfg.draft
                wbytes = 2 * (d.n_layers * (4 * d.d_model ** 2 + 2 * d.d_model * d.d_ff) + 2 * cfg.patch * d.d_model)
                # (K steps per launch; the last rounds of a decode run fewer, so this is a slight overestimate)
                out[name]["achieved_gbs_per_cu"] = wbytes * cfg.K / (ms * 1e-3 / n) / 1e9
            continue
        hbm = name in ("attn", "accept", "route")
        achieved = work / (ms * 1e-3) / (1e9 if hbm else 1e12)
        peak = HBM_PEAK if hbm else PEAK[dtype]
        out[name] = dict(bound="hbm" if hbm else "mfma", achieved=achieved, peak=peak, unit="GB/s" if hbm else "TFLOP/s",
                         frac=achieved / peak, launches=n, avg_us=ms * 1e3 / n, total_ms=ms,
                         traffic=TRAFFIC.get(workload, {}).get(name))
        # the GEMMs of this size sit near the ridge (intensity ~ 300 flop per HBM byte): besides the
        # MFMA fraction, the measured HBM bytes per launch against the memory peak
        if out[name]["traffic"]:
            out[name]["hbm_frac_of_traffic"] = out[name]["traffic"] / (ms * 1e-3 / n) / 1e9 / HBM_PEAK
    return out


def measured_peaks(torch, tsd):
    """What this machine delivers to the simplest possible kernels: the library's register-only MFMA
    loop (bf16 32x32x16, every wavefront slot of every CU busy) and its plain 256 MiB copy kernel.
    Reported beside the published peaks the roofline fractions are quoted against."""
    def ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    blocks, iters = 256 * 8, 20000
    sink = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    t = ms(lambda: tsd.bench_mfma(blocks, iters, sink), 3)
    mfma = blocks * 4 * iters * 4 * 2.0 * 32 * 32 * 16 / (t * 1e-3) / 1e12
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")      # 256 MiB
    dst = torch.empty_like(src)
    t = ms(lambda: tsd.bench_copy(dst, src), 5)
    copy = 2.0 * src.numel() * 4 / (t * 1e-3) / 1e9
    return {"mfma_bf16_tflops": mfma, "hbm_copy_gbs": copy}


def cpu_baseline(case, n_series, batch_sync=False, **oracle_kw):
    """The oracle, as it stands, on a bounded sample: n_series series, whole horizon,
    single-pass mode, one process (numpy's BLAS threads).  The only place the oracle is used."""
    from oracle import tsd_oracle as orc
    c = case.cfg
    Wt, Wd = orc.as_f64(case.wt), orc.as_f64(case.wd)
    t0 = time.perf_counter()
    if batch_sync:   # the sample decodes as one synchronised batch of its own
        orc.forecast_spec_sync(Wt, c.target, Wd, c.draft, case.context[:n_series], c.patch, c.horizon, c.K, c.sigma,
                               c.sigma, case.seed, **oracle_kw)
    else:
        for b in range(n_series):
            orc.forecast_spec(Wt, c.target, Wd, c.draft, case.context[b], c.patch, c.horizon, c.K, c.sigma,
                              c.sigma, case.seed, b, **oracle_kw)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    return dict(value=n_series * c.horizon / dt, unit="forecast steps/s", cores=cores, kind="oracle",
                sample=f"{n_series} of {c.batch} series, whole horizon of {c.horizon} steps, "
                       f"{'single-pass' if oracle_kw.get('single_pass', True) else 'per-prefix'} oracle"
                       f"{', threshold rule' if oracle_kw.get('rule') == 'threshold' else ''}"
                       f"{', batch-synchronised' if batch_sync else ''}, {dt:.1f} s")


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2511_18191_amd as tsd
    import synth

    if a.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")      # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(5):
            tsd.bench_copy(dst, src)
        torch.cuda.synchronize()
        assert torch.equal(dst[:1024], src[:1024])
        del src, dst

    case = synth.Inputs(a.config, sigma=a.sigma, B=a.batch)
    c = case.cfg
    flags = (tsd.TSD_FLAG_SAMPLE_PROPOSALS if a.sample_proposals else 0) | (tsd.TSD_FLAG_NAIVE_VERIFY if a.naive_verify else 0)
    flags |= (tsd.TSD_FLAG_THRESHOLD_RULE if a.threshold_rule else 0) | (tsd.TSD_FLAG_BATCH_SYNC if a.batch_sync else 0)
    flags |= {"auto": 0, "on": tsd.TSD_FLAG_FUSED_DRAFT, "off": tsd.TSD_FLAG_NO_FUSED_DRAFT}[a.fused_draft]
    sess = tsd.session_for(case, flags=flags, fallback_r=a.fallback_r)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sess.prefill(case.context, c.n_ctx, c.horizon)
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - t0) * 1e3

    for _ in range(a.warmup):
        decode_spec(sess)
    rounds = decode_spec(sess)
    st = sess.get_stats()
    t_spec = timed(torch, lambda: decode_spec(sess), a.steps)
    for _ in range(max(1, a.warmup // 2)):
        decode_target_only(sess, c.T)
    t_base = timed(torch, lambda: decode_target_only(sess, c.T), a.steps)
    ph = phase_times(torch, sess)

    fam = kernel_rooflines(sess, c.dtype, max(2, a.steps // 4), c.name if a.sigma is None and a.batch is None else None, cfg=c)
    # the one-launch draft kernel is listed with its own bound below; the headline roofline goes to the
    # largest family that one of the two published peaks (MFMA, HBM) bounds
    dominant = max((k for k in fam if k != "draft"), key=lambda k: fam[k]["total_ms"])
    peaks = measured_peaks(torch, tsd)

    alpha = st["accepted"] / max(1, st["tested"])
    mean_L = st["committed"] / max(1, st["rounds"])
    cc = ph["draft"] / c.K / ph["target_step"]
    v = (ph["verify"] + ph["accept"]) / ph["target_step"]
    out = {
        "metric": "forecast steps/s (batched spec decode) + speedup vs target-only AR decode",
        "value": c.batch * c.horizon / t_spec,
        "unit": "forecast steps/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": t_spec * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": c.dtype, "data": "synthetic",
        "config": {"workload": f"{c.name}: B={c.batch} P={c.patch} N={c.n_ctx} H={c.horizon} K={c.K} sigma={c.sigma} "
                               f"target {c.target.n_layers}L/d{c.target.d_model} draft {c.draft.n_layers}L/d{c.draft.d_model}",
                   "step": "reset to post-prefill state + speculative rounds until all series reach the horizon",
                   "ablation": {"sample_proposals": a.sample_proposals, "fallback_r": a.fallback_r, "naive_verify": a.naive_verify,
                                "threshold_rule": a.threshold_rule, "batch_sync": a.batch_sync, "fused_draft": a.fused_draft}},
        "speedup_vs_target_only": t_base / t_spec,
        "target_only_steps_per_s": c.batch * c.horizon / t_base,
        "target_only_ms": t_base * 1e3,
        "prefill_ms": prefill_ms,
        "rounds_per_decode": rounds,
        "acceptance": alpha, "mean_committed_per_round": mean_L,
        "phase_ms": ph, "c": cc, "v": v,
        "predicted_speedup_eq8": tsd.law.speedup(alpha, c.K, cc, v),
        "near_ties": st["near_ties"],
        # committed patches per unit time against one patch per target step (what Eq. 8 predicts)
        "patch_rate_speedup": mean_L * ph["target_step"] / (ph["draft"] + ph["verify"] + ph["accept"]),
        "roofline": dict({k: v for k, v in fam[dominant].items()
                          if k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "hbm_frac_of_traffic")},
                         kernel=dominant, avg_us=fam[dominant]["avg_us"], launches=fam[dominant]["launches"]),
        "kernel_families": fam,
        "measured_peaks": peaks,
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case, min(a.cpu_series, c.batch), sample_proposals=a.sample_proposals,
                                           fallback_r=a.fallback_r, single_pass=not a.naive_verify,
                                           rule="threshold" if a.threshold_rule else "ratio", batch_sync=a.batch_sync)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
