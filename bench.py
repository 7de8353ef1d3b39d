#!/usr/bin/env python3
"""Benchmark of the speculative-decoding hot path on one MI355X.

A step is one whole speculative decode of the batch: reset to the post-prefill state, then
rounds (draft proposal, single-pass verification, acceptance/commit/rollback) until every series
has its horizon.  Inputs (weights, KV cache of the context) are resident in HBM before the
timed region.  Prints ONE JSON line: the headline workload (default cfg3, the largest configuration
that one GPU holds and the one whose GEMMs and attention the MFMA / HBM rooflines bound), its dominant
kernel family's roofline, the CPU oracle on a bounded sample of the same workload, and a `configs`
block with the same figures for every one of the five configurations.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3] [--sigma 1.0] [--only]
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

ALL_CONFIGS = ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--only", action="store_true", help="skip the `configs` block (the other four configurations)")
    ap.add_argument("--sigma", type=float, default=None)
    ap.add_argument("--batch", type=int, default=None, help="series in the batch (default: the configuration's; other sizes are side experiments)")
    ap.add_argument("--sample-proposals", action="store_true", help="ablation: x_i = mu_q + sigma_q eps")
    ap.add_argument("--fallback-r", type=float, default=0.0, help="ablation: fallback / bonus noise scale")
    ap.add_argument("--naive-verify", action="store_true", help="ablation: one target pass per prefix")
    ap.add_argument("--threshold-rule", action="store_true", help="variant: accept iff ||x - mu_p||_d^2 <= sigma^2")
    ap.add_argument("--batch-sync", action="store_true", help="variant: all series keep the batch's smallest accepted count")
    ap.add_argument("--fused-draft", choices=["auto", "on", "off"], default="auto",
                    help="the draft phase as one launch: where the library picks it (auto), wherever supported (on), never (off)")
    ap.add_argument("--no-wide", action="store_true", help="A/B: never the wide-tile direct-to-LDS GEMM kernels (same bits)")
    ap.add_argument("--drain-every", type=int, default=0,
                    help="wait for the stream after this many target-only steps (for runs under a counter-collecting profiler, "
                         "which stalls when thousands of launches are queued without a host wait)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-workers", type=int, default=0, help="oracle worker processes (default: the CPUs this process may use, at most 16)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="the oracle keeps taking series until about this much wall time has passed")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB copy kernel 5 times (known traffic, to scale profiler memory counters) and "
                         "bracket the kernel-by-kernel timing pass with two marker copies of 28672 bytes")
    return ap.parse_args()


def log(msg):
    """Progress on stderr (the JSON line on stdout stays alone): long runs under a profiler show where they are."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def decode_spec(sess):
    sess.reset_decode()
    return sess.run_rounds()[0]   # rounds until every series has its horizon (the loop lives in the library)


DRAIN_EVERY = 0   # --drain-every: wait for the stream after this many target-only steps (0: never)


def decode_target_only(sess, T):
    sess.reset_decode()
    for i in range(T):
        sess.target_step()
        if DRAIN_EVERY and (i + 1) % DRAIN_EVERY == 0:
            sess.sync()


def timed(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()       # waits for every stream of the device, the session's included
    return (time.perf_counter() - t0) / steps


def phase_times(torch, sess, reps=10):
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


PEAK = {"bf16": 2500.0, "fp32": 157.3}   # dense MFMA bf16 / vector fp32, TFLOP/s
HBM_PEAK = 8000.0                        # GB/s


def library_sources_hash():
    """Identifies the kernel sources a profile was taken with (profiles/traffic_*.txt carry the same value)."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2511_18191_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".h")):
            h.update(f.encode())
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per launch of each kernel family from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of
    this workload (profiles/traffic_<workload>_bench.txt: commands, raw values, copy-kernel scale factors).  Used
    only when that summary was taken with the kernel sources as they are now; otherwise no traffic is reported."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}_bench.txt")
    if workload is None or not os.path.exists(path):
        return {}, "no committed counter summary for this workload"
    text = open(path).read()
    m = re.search(r"kernel sources: ([0-9a-f]{16})", text)
    if not m or m.group(1) != library_sources_hash():
        return {}, "the committed counter summary is of other kernel sources"
    if "## timing pass only" in text:      # the launch mix `achieved` is computed on, where the summary has it apart
        text = text[text.index("## timing pass only"):]
    out = {}
    for row in re.findall(r"^\| *([a-z]+(?:\[[0-9a-z]+\])?) *\|(?:[^|]*\|){5} *([0-9.]+) *\|", text, flags=re.M):
        out[row[0]] = int(round(float(row[1]) * 1e6))
    return out, os.path.relpath(path, ROOT)


def attention_bytes_per_decode(sess, c, fused_draft):
    """The K and V rows every attention launch of one speculative decode has to read, exactly, in launch order: one
    more decode, round by round, reading every series' committed count before each round.  A series with `len` cached
    tokens reads len + nq rows of K and of V in a pass of nq new tokens (the verification: nq = positions + 1; the
    draft, unless it runs as one fused launch: 2 tokens from position len - 1, then one per step), plus its q rows and
    output rows.  (The library's own tally books every launch at the shortest history a series can have.)
    Returns a list of (model, bytes) per launch."""
    import numpy as np
    es = 2 if c.dtype == "bf16" else 4
    sess.reset_decode()
    out = []
    active = c.batch
    while active > 0:
        committed = sess.get_state()["committed"].cpu().numpy().astype(np.int64)
        on = committed < c.T
        ln = (c.n_ctx - 1 + committed)[on].astype(np.float64)
        kr = int(min(c.K, (c.T - committed[on]).max()))
        n = float(on.sum())
        t, d = c.target, c.draft
        if not fused_draft:
            for i in range(1, kr + 1):          # step 1 reads len + 1 rows (two new tokens from len - 1), step i >= 2 len + i
                rows, nq = (ln + i).sum(), (2 if i == 1 else 1)
                out += [(1, d.d_model * es * (2.0 * rows + 2.0 * nq * n))] * d.n_layers
        out += [(0, t.d_model * es * (2.0 * (ln + kr + 1).sum() + 2.0 * (kr + 1) * n))] * t.n_layers
        sess.round()
        active = sess.num_active()
    return out


# --copy-calibration: a callable that launches one small copy of a size nothing else uses (28672 bytes: 7 workgroups),
# before and after the kernel-by-kernel timing pass, so that a profiler's per-dispatch records of exactly that pass
# (the launch mix `achieved` is computed on) can be told from the rest of the run
MARK = None


TILE_LABEL = {128: "128x128", 64: "64x64", 464: "64x64k4", 16: "skinny", 2256: "w256x128", 2128: "w128x128"}


def kernel_rooflines(sess, dtype, steps, traffic, cfg=None):
    """Per kernel (family and, for the GEMM families, the tile variant the launcher picked): HIP-event time of
    every launch during `steps` speculative decodes (kernel-by-kernel launches on the session's stream, every
    launch bracketed by two events) and the algorithmic work they did."""
    from paper_2511_18191_amd.binding import KERNEL_CLASSES
    if MARK:
        MARK()
    sess.profile_begin(len(KERNEL_CLASSES))       # every family at once
    for _ in range(steps):
        decode_spec(sess)
    sess.profile_end()
    if MARK:
        MARK()
    launches = sess.profile_launches()
    fused = any(KERNEL_CLASSES[r["kernel_class"]] == "draft" for r in launches)
    exact = attention_bytes_per_decode(sess, cfg, fused) if cfg is not None else []
    attn_recs = [r for r in launches if KERNEL_CLASSES[r["kernel_class"]] == "attn"]
    if exact and len(attn_recs) == steps * len(exact) and all(r["model"] == m for r, (m, _) in zip(attn_recs, exact * steps)):
        for r, (_, nbytes) in zip(attn_recs, exact * steps):
            r["floor_work"], r["work"] = r["work"], nbytes    # the rows actually cached, not the shortest possible history
    groups = {}
    for r in launches:
        name = KERNEL_CLASSES[r["kernel_class"]]
        if name == "attn":
            key = "attn[%s]" % {0: "target", 1: "draft"}.get(r["model"], "?")
        elif r["tile"] in TILE_LABEL and name not in ("accept", "route", "draft"):
            key = f"{name}[{TILE_LABEL[r['tile']]}]"
        else:
            key = name
        g = groups.setdefault(key, dict(family=name, n=0, ms=0.0, work=0.0, rows=0, floor=0.0, big=None))
        g["n"] += 1; g["ms"] += r["ms"]; g["work"] += r["work"]; g["rows"] += r["M"]; g["floor"] += r.get("floor_work", 0.0)
        # the launches of the group's largest shape (full-batch passes), kept apart
        if g["big"] is None or r["M"] > g["big"]["M"]:
            g["big"] = dict(M=r["M"], n=0, ms=0.0, work=0.0)
        if r["M"] == g["big"]["M"]:
            g["big"]["n"] += 1; g["big"]["ms"] += r["ms"]; g["big"]["work"] += r["work"]
    out = {}
    for key, g in groups.items():
        name, n, ms, work = g["family"], g["n"], g["ms"], g["work"]
        if name == "draft":
            # one launch runs all K draft steps; every workgroup streams the draft's weights once per step
            # through its compute unit's vector-memory path (64 B/clk at 2.4 GHz = 153.6 GB/s per unit)
            out[key] = dict(bound="cu_stream", launches=n, avg_us=ms * 1e3 / n, total_ms=ms,
                            mfma_tflops=work / (ms * 1e-3) / 1e12, peak_gbs_per_cu=153.6, unit="GB/s per CU",
                            traffic=traffic.get(key))
            if cfg is not None:
                d = cfg.draft
                wbytes = 2 * (d.n_layers * (4 * d.d_model ** 2 + 2 * d.d_model * d.d_ff) + 2 * cfg.patch * d.d_model)
                # (K steps per launch; the last rounds of a decode run fewer, so this is a slight overestimate)
                out[key]["achieved_gbs_per_cu"] = wbytes * cfg.K / (ms * 1e-3 / n) / 1e9
            continue
        hbm = name in ("attn", "accept", "route")
        floor_work = g["floor"] if g["floor"] > 0 else None
        achieved = work / (ms * 1e-3) / (1e9 if hbm else 1e12)
        peak = HBM_PEAK if hbm else PEAK[dtype]
        out[key] = dict(bound="hbm" if hbm else ("mfma" if dtype == "bf16" else "alu"), achieved=achieved, peak=peak,
                        unit="GB/s" if hbm else "TFLOP/s", frac=achieved / peak, launches=n, avg_us=ms * 1e3 / n,
                        total_ms=ms, avg_rows=g["rows"] / n, work_per_launch=work / n, traffic=traffic.get(key))
        big = g["big"]
        if big and big["n"] < n:   # the group's largest launches alone (the full-batch passes)
            a_big = big["work"] / (big["ms"] * 1e-3) / (1e9 if hbm else 1e12)
            out[key]["largest_launches"] = dict(rows=big["M"], launches=big["n"], avg_us=big["ms"] * 1e3 / big["n"],
                                                achieved=a_big, frac=a_big / peak)
        if floor_work is not None:
            out[key]["achieved_at_shortest_history"] = floor_work / (ms * 1e-3) / 1e9
        if out[key]["traffic"]:
            out[key]["hbm_frac_of_traffic"] = out[key]["traffic"] / (ms * 1e-3 / n) / 1e9 / HBM_PEAK
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


def batch_level_prediction(torch, sess, case, c, t_base):
    """The whole-batch decode time the capped-geometric law predicts once the batch's lock-step is modelled, and the
    block size with the shortest predicted decode (planner.batch_decode_model; measured round times by active count).
    Leaves the handle prefilled with the whole batch again."""
    from paper_2511_18191_amd import planner
    per = sess.get_series_stats().cpu().numpy()                               # of the last decode: rounds, tested, accepted, ...
    cost = planner.round_times(sess, case.context, c.n_ctx, c.horizon, c.K)
    out = planner.batch_decode_model(per[:, 1], per[:, 2], cost, c.K, c.T)
    for name in ("pooled_acceptance", "per_series_acceptance"):
        out[name]["predicted_speedup_vs_target_only"] = t_base * 1e3 / out[name]["predicted_ms"]
    return out


# ---- the CPU oracle on a bounded sample: runs BEFORE anything touches the GPU (forked workers) -------------
_ORC = {}


def _oracle_series(b):
    """One series, whole horizon, in a worker process (BLAS held to one thread: the threading is over series)."""
    o = _ORC
    c = o["case"].cfg
    from threadpoolctl import threadpool_limits
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        o["orc"].forecast_spec(o["Wt"], c.target, o["Wd"], c.draft, o["case"].context[b], c.patch, c.horizon, c.K, c.sigma,
                               c.sigma, o["case"].seed, b, **o["kw"])
        return time.perf_counter() - t0


def cpu_baseline(case, workers, seconds, batch_sync=False, **oracle_kw):
    """The oracle, as it stands, timed on this machine's host cores on a bounded sample of the workload: whole
    series (full horizon, single-pass mode), one per worker process at a time, until about `seconds` have
    passed.  The only place the benchmark uses the oracle."""
    import multiprocessing as mp
    from oracle import tsd_oracle as orc
    c = case.cfg
    Wt, Wd = orc.as_f64(case.wt), orc.as_f64(case.wd)
    if batch_sync:   # the synchronised loop couples the series of a batch: one process, the sample as its own batch
        n = min(c.batch, 8)
        t0 = time.perf_counter()
        orc.forecast_spec_sync(Wt, c.target, Wd, c.draft, case.context[:n], c.patch, c.horizon, c.K, c.sigma, c.sigma,
                               case.seed, **oracle_kw)
        dt = time.perf_counter() - t0
        return dict(value=n * c.horizon / dt, unit="forecast steps/s", cores=1, kind="oracle",
                    sample=f"{n} of {c.batch} series as one synchronised batch, whole horizon of {c.horizon} steps, {dt:.1f} s")
    _ORC.update(case=case, Wt=Wt, Wd=Wd, orc=orc, kw=oracle_kw)
    workers = max(1, min(workers, c.batch))
    done, t0 = 0, time.perf_counter()
    with mp.get_context("fork").Pool(workers) as pool:       # forked: the float64 weights are shared, not copied
        while done < c.batch:
            take = list(range(done, min(c.batch, done + workers)))
            per_series = pool.map(_oracle_series, take, chunksize=1)
            done += len(take)
            if time.perf_counter() - t0 >= seconds:
                break
    dt = time.perf_counter() - t0
    _ORC.clear()
    return dict(value=done * c.horizon / dt, unit="forecast steps/s", cores=workers, kind="oracle",
                sample=f"{done} of {c.batch} series of {c.name}, whole horizon of {c.horizon} steps, "
                       f"{'single-pass' if oracle_kw.get('single_pass', True) else 'per-prefix'} oracle"
                       f"{', threshold rule' if oracle_kw.get('rule') == 'threshold' else ''}, one series per worker process "
                       f"(BLAS single-threaded), {dt:.1f} s wall, last batch {max(per_series):.1f} s per series")


def run_config(torch, tsd, synth, a, name, steps, warmup, fam_steps, flags, case=None, full=True):
    """One configuration: speculative decode, target-only decode, phases, kernel families."""
    if case is None:
        case = synth.Inputs(name, sigma=a.sigma if full else None, B=a.batch if full else None)
    c = case.cfg
    log(f"{c.name}: weights to the device")
    sess = tsd.session_for(case, flags=flags, fallback_r=a.fallback_r if full else 0.0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sess.prefill(case.context, c.n_ctx, c.horizon)
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - t0) * 1e3
    log(f"{c.name}: prefill {prefill_ms:.1f} ms; speculative decodes")
    for _ in range(warmup):
        decode_spec(sess)
    rounds = decode_spec(sess)
    st = sess.get_stats()
    t_spec = timed(torch, lambda: decode_spec(sess), steps)
    log(f"{c.name}: {t_spec * 1e3:.2f} ms per speculative decode; target-only decodes")
    for _ in range(max(1, warmup // 2)):
        decode_target_only(sess, c.T)
    t_base = timed(torch, lambda: decode_target_only(sess, c.T), steps)
    log(f"{c.name}: {t_base * 1e3:.2f} ms per target-only decode; phases")
    ph = phase_times(torch, sess, reps=10 if full else 5)
    alpha = st["accepted"] / max(1, st["tested"])
    batch_pred, planned = None, None
    if flags == 0:
        log(f"{c.name}: round times by active count, batch-level prediction")
        decode_spec(sess)                                                     # per-series counters of a whole decode at the configured K
        batch_pred = batch_level_prediction(torch, sess, case, c, t_base)
        batch_pred.update(measured_ms=t_spec * 1e3, measured_rounds=rounds, measured_speedup_vs_target_only=t_base / t_spec)
    # the method's own choice of block size (Proposition "Marginal-gain condition for K"), two ways: Eq. 8 maximised
    # over the measured cost table c(K), v(K) (committed patches per unit time of one series), and the shortest predicted
    # decode of the whole batch (the lock-step model above); a decode at each
    if c.K > 1 and flags == 0:
        from paper_2511_18191_amd import planner
        log(f"{c.name}: cost table for K = 1..{c.K}")
        costs = planner.cost_table(sess, c.K, reps=4)
        planned = {"v_of_K": {str(k): round(costs[k]["v"], 3) for k in costs}, "c_of_K": {str(k): round(costs[k]["c"], 4) for k in costs}}
        timed_at = {c.K: (t_spec, st)}
        for rule, k_star in (("eq8_over_measured_cost_table", planner.plan(alpha, costs, min(2, c.K))["k_table"]),
                             ("shortest_predicted_batch_decode", batch_pred["best_block_size"])):
            if k_star not in timed_at:
                sess.set_block_size(k_star)
                decode_spec(sess)
                st_k = sess.get_stats()
                timed_at[k_star] = (timed(torch, lambda: decode_spec(sess), max(2, steps // 2)), st_k)
                sess.set_block_size(c.K)
            t_k, st_k = timed_at[k_star]
            planned[rule] = {"K": k_star, "value": c.batch * c.horizon / t_k, "ms_per_step": t_k * 1e3, "speedup_vs_target_only": t_base / t_k,
                             "acceptance": st_k["accepted"] / max(1, st_k["tested"]),
                             "mean_committed_per_round": st_k["committed"] / max(1, st_k["rounds"])}
    log(f"{c.name}: kernel-by-kernel timing pass")
    standard = full and a.sigma is None and a.batch is None and flags == 0 and a.fallback_r == 0.0
    traffic, traffic_src = measured_traffic(c.name if (standard or not full) else None)
    fam = kernel_rooflines(sess, c.dtype, fam_steps, traffic, cfg=c)
    sess.close()
    # the one-launch draft kernel is listed with its own bound; the headline roofline goes to the largest
    # family that one of the published peaks (MFMA, HBM) bounds
    dominant = max((k for k in fam if fam[k]["bound"] != "cu_stream"), key=lambda k: fam[k]["total_ms"])
    mean_L = st["committed"] / max(1, st["rounds"])
    cc = ph["draft"] / c.K / ph["target_step"]
    v = (ph["verify"] + ph["accept"]) / ph["target_step"]
    rec = {
        "workload": f"{c.name}: B={c.batch} P={c.patch} N={c.n_ctx} H={c.horizon} K={c.K} sigma={c.sigma} "
                    f"target {c.target.n_layers}L/d{c.target.d_model}{'/%dx top-%d experts' % (c.target.n_experts, c.target.top_k) if c.target.n_experts else ''} "
                    f"draft {c.draft.n_layers}L/d{c.draft.d_model}",
        "dtype": c.dtype,
        "value": c.batch * c.horizon / t_spec, "unit": "forecast steps/s", "ms_per_step": t_spec * 1e3, "steps": steps,
        "speedup_vs_target_only": t_base / t_spec,
        "target_only_steps_per_s": c.batch * c.horizon / t_base, "target_only_ms": t_base * 1e3,
        "prefill_ms": prefill_ms, "rounds_per_decode": rounds,
        "acceptance": alpha, "mean_committed_per_round": mean_L,
        "phase_ms": ph, "c": cc, "v": v,
        "predicted_speedup_eq8": tsd.law.speedup(alpha, c.K, cc, v),
        # committed patches per unit time against one patch per target step: what Eq. 8 predicts (the batch-level
        # figure above also pays for rounds in which only the slowest series are still decoding)
        "patch_rate_speedup": mean_L * ph["target_step"] / (ph["draft"] + ph["verify"] + ph["accept"]),
        "near_ties": st["near_ties"],
        "planned_block_size": planned,
        "batch_level_prediction": batch_pred,
        "roofline": dict({k: v_ for k, v_ in fam[dominant].items()
                          if k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "hbm_frac_of_traffic")},
                         kernel=dominant, avg_us=fam[dominant]["avg_us"], launches=fam[dominant]["launches"],
                         traffic_source=traffic_src),
        "kernel_families": fam,
    }
    return rec


def main():
    a = parse()
    global DRAIN_EVERY, MARK
    DRAIN_EVERY = a.drain_every
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import synth

    # The oracle's leg first, in forked worker processes, before this process has touched the GPU.
    case = synth.Inputs(a.config, sigma=a.sigma, B=a.batch)
    cpu = None
    if not a.no_cpu_baseline:
        try:
            avail = len(os.sched_getaffinity(0))
        except AttributeError:
            avail = os.cpu_count() or 1
        workers = a.cpu_workers or min(16, avail)
        log(f"oracle on {workers} worker processes, about {a.cpu_seconds:.0f} s")
        cpu = cpu_baseline(case, workers, a.cpu_seconds, sample_proposals=a.sample_proposals, fallback_r=a.fallback_r,
                           single_pass=not a.naive_verify, rule="threshold" if a.threshold_rule else "ratio",
                           batch_sync=a.batch_sync)

    import torch
    import paper_2511_18191_amd as tsd

    if a.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")      # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(5):
            tsd.bench_copy(dst, src)
        torch.cuda.synchronize()
        assert torch.equal(dst[:1024], src[:1024])
        del src, dst
        m_src = torch.ones(7 * 256 * 4, dtype=torch.float32, device="cuda")
        m_dst = torch.empty_like(m_src)

        def mark():
            torch.cuda.synchronize()
            tsd.bench_copy(m_dst, m_src)
            torch.cuda.synchronize()
        MARK = mark

    flags = (tsd.TSD_FLAG_SAMPLE_PROPOSALS if a.sample_proposals else 0) | (tsd.TSD_FLAG_NAIVE_VERIFY if a.naive_verify else 0)
    flags |= (tsd.TSD_FLAG_THRESHOLD_RULE if a.threshold_rule else 0) | (tsd.TSD_FLAG_BATCH_SYNC if a.batch_sync else 0)
    flags |= {"auto": 0, "on": tsd.TSD_FLAG_FUSED_DRAFT, "off": tsd.TSD_FLAG_NO_FUSED_DRAFT}[a.fused_draft]
    flags |= tsd.TSD_FLAG_NO_WIDE_GEMM if a.no_wide else 0
    head = run_config(torch, tsd, synth, a, a.config, a.steps, a.warmup, max(2, a.steps // 4), flags, case=case)
    del case
    peaks = measured_peaks(torch, tsd)

    out = {
        "metric": "forecast steps/s (batched spec decode) + speedup vs target-only AR decode",
        "value": head["value"], "unit": "forecast steps/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"],
                   "step": "reset to post-prefill state + speculative rounds until all series reach the horizon",
                   "ablation": {"sample_proposals": a.sample_proposals, "fallback_r": a.fallback_r, "naive_verify": a.naive_verify,
                                "threshold_rule": a.threshold_rule, "batch_sync": a.batch_sync, "fused_draft": a.fused_draft,
                                "no_wide_gemm": a.no_wide}},
    }
    out.update({k: head[k] for k in ("speedup_vs_target_only", "target_only_steps_per_s", "target_only_ms", "prefill_ms",
                                     "rounds_per_decode", "acceptance", "mean_committed_per_round", "phase_ms", "c", "v",
                                     "predicted_speedup_eq8", "near_ties", "patch_rate_speedup", "planned_block_size",
                                     "batch_level_prediction", "roofline", "kernel_families")})
    out["measured_peaks"] = peaks
    if cpu is not None:
        out["cpu_baseline"] = cpu
    if not a.only:
        # the five configurations, each in the deployed scheme (no ablation flags), fewer repetitions
        short = ("workload", "dtype", "value", "ms_per_step", "steps", "speedup_vs_target_only", "target_only_ms", "rounds_per_decode",
                 "acceptance", "mean_committed_per_round", "phase_ms", "c", "v", "predicted_speedup_eq8", "patch_rate_speedup",
                 "planned_block_size", "batch_level_prediction", "roofline")
        block = {}
        for name in ALL_CONFIGS:
            if name == a.config and flags == 0 and a.sigma is None and a.batch is None and a.fallback_r == 0.0:
                rec = head
            else:
                n = 3 if name in ("cfg3", "cfg5") else 5
                rec = run_config(torch, tsd, synth, a, name, n, 1, 1, 0, full=False)
            block[name] = {k: rec[k] for k in short}
            block[name]["families"] = {k: {kk: f[kk] for kk in ("bound", "achieved", "frac", "avg_us", "launches", "unit") if kk in f}
                                       for k, f in rec["kernel_families"].items()}
        out["configs"] = block
    print(json.dumps(out))


if __name__ == "__main__":
    main()
