"""Component ablation on one GPU, one row per replaced component (the layout of the paper's
component-ablation table): acceptance, deviation from the target-only forecast, speed.

    python -m paper_2511_18191_amd.ablate --config cfg2 --sigma 1.0

Rows: the full rule; without the 1/d tempering; sampled proposals x_i ~ q instead of the mean;
fallback noise r = sigma instead of the clean target mean; one target pass per prefix instead of
single-pass verification; and the standalone variant of the paper's TiRex table: the deterministic
threshold ||x - mu_p||_d^2 <= sigma^2 with batch-synchronised commits, alone and on top of
per-prefix verification.  There is no trained model or dataset here, so "accuracy" is the mean
energy per dimension of (forecast - target-only forecast) in normalised units: the quantity the
deterministic fidelity bound (Eq. 9) caps at 2 sigma^2 / e per committed patch for the full rule.
Prints a markdown table.
"""
import argparse
import sys

import numpy as np

import synth

from .binding import (TSD_FLAG_BATCH_SYNC, TSD_FLAG_NAIVE_VERIFY, TSD_FLAG_NO_FUSED_DRAFT, TSD_FLAG_NO_TEMPERING, TSD_FLAG_SAMPLE_PROPOSALS,
                      TSD_FLAG_THRESHOLD_RULE, session_for)
from .sweep import _decode_spec, _decode_target, _time


def run(inputs, flags, fallback_r, reps):
    import torch
    c = inputs.cfg
    sess = session_for(inputs, flags=flags, fallback_r=fallback_r)
    sess.prefill(inputs.context, c.n_ctx, c.horizon)
    _decode_spec(sess)
    y = sess.get_forecast().cpu().numpy()
    st = sess.get_stats()
    t_spec = _time(torch, lambda: _decode_spec(sess), reps)
    _decode_target(sess, c.T)
    y_t = sess.get_forecast().cpu().numpy()
    t_base = _time(torch, lambda: _decode_target(sess, c.T), reps)
    sess.close()
    sd = np.sqrt(inputs.context.astype(np.float64).var(axis=1) + 1e-5)[:, None]
    dev = float((((y - y_t) / sd) ** 2).mean())
    return dict(accept=st["accepted"] / max(1, st["tested"]), L=st["committed"] / max(1, st["rounds"]), dev=dev,
                t_spec=t_spec * 1e3, t_base=t_base * 1e3)


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--sigma", type=float, default=None)
    ap.add_argument("--K", type=int, default=None)
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args(argv)
    inputs = synth.Inputs(a.config, sigma=a.sigma, K=a.K)
    c = inputs.cfg
    rows = [("full rule", 0, 0.0), ("w/o 1/d tempering", TSD_FLAG_NO_TEMPERING, 0.0),
            ("w/o mean proposal (x_i ~ q)", TSD_FLAG_SAMPLE_PROPOSALS, 0.0), ("w/o clean fallback (r = sigma)", 0, c.sigma),
            ("w/o single-pass verification", TSD_FLAG_NAIVE_VERIFY, 0.0),
            ("full rule, draft phase kernel by kernel", TSD_FLAG_NO_FUSED_DRAFT, 0.0),
            ("batch-synchronised commits", TSD_FLAG_BATCH_SYNC, 0.0),
            ("threshold rule", TSD_FLAG_THRESHOLD_RULE, 0.0),
            ("threshold rule, batch-synchronised", TSD_FLAG_THRESHOLD_RULE | TSD_FLAG_BATCH_SYNC, 0.0),
            ("threshold rule, batch-synchronised, per-prefix verification",
             TSD_FLAG_THRESHOLD_RULE | TSD_FLAG_BATCH_SYNC | TSD_FLAG_NAIVE_VERIFY, 0.0)]
    print(f"{c.name}: B={c.batch} P={c.patch} K={c.K} sigma={c.sigma:g} H={c.horizon}; fidelity cap of the full rule "
          f"2 sigma^2/e = {2 * c.sigma ** 2 / np.e:.3f}\n")
    print("| configuration | accept | patches/round | deviation from target-only | spec ms | target-only ms | speedup |")
    print("|---|---|---|---|---|---|---|")
    for name, flags, r in rows:
        m = run(inputs, flags, r, a.reps)
        print(f"| {name} | {100 * m['accept']:.1f} % | {m['L']:.2f} | {m['dev']:.4f} | {m['t_spec']:.2f} | {m['t_base']:.2f} | "
              f"{m['t_base'] / m['t_spec']:.2f}x |", flush=True)


if __name__ == "__main__":
    sys.exit(main())
