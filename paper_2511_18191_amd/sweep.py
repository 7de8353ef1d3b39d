"""Block-size and temperature sweeps on one GPU, reported next to the paper's throughput law.

    python -m paper_2511_18191_amd.sweep --config cfg4 --K 1 2 3 4 5 6 7 8 --series 8
    python -m paper_2511_18191_amd.sweep --config cfg2 --sigma 0.5 1 2
    python -m paper_2511_18191_amd.sweep --config cfg3 --calibrate 0.7 0.9

--calibrate finds, by bisection on whole decodes, the temperature at which the measured acceptance
(accepted / tested) hits each given rate, and sweeps those temperatures: random-init models need not
reject anything at sigma = 1, and a workload whose rejection path carries no weight measures
half of the round.

For every point: speculative decode time, matched target-only time, acceptance (accepted / tested),
committed patches per series-round against Eq. 7 at the measured acceptance, measured cost ratios
c (draft call / target step) and v ((verify + accept) / target step), Eq. 8's predicted speedup
against the measured committed-patch-rate speedup, and whether one more position would pay
(marginal criterion).  Prints a markdown table.
"""
import argparse
import sys
import time

import synth

from . import law
from .binding import session_for


def _decode_spec(sess):
    sess.reset_decode()
    return sess.run_rounds()[0]


def _decode_target(sess, T):
    sess.reset_decode()
    for _ in range(T):
        sess.target_step()


def _time(torch, fn, reps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def _phase(torch, sess, fn, before, reps=10):
    tot = 0.0
    for _ in range(reps):
        sess.reset_decode()
        before()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(sess.stream); fn(); b.record(sess.stream)
        torch.cuda.synchronize()
        tot += a.elapsed_time(b)
    return tot / reps


def calibrate_sigma(inputs, target, lo=0.02, hi=16.0, tol=0.004, iters=24):
    """Temperature (sigma_p = sigma_q) at which a whole speculative decode of `inputs` accepts the
    fraction `target` of its tested proposals; the ratio rule's acceptance rises with sigma, so a
    bisection on log sigma finds it.  Returns (sigma, acceptance there)."""
    c = inputs.cfg
    sess = session_for(inputs)
    sess.prefill(inputs.context, c.n_ctx, c.horizon)

    def rate(sigma):
        sess.set_sigma(sigma)
        _decode_spec(sess)
        st = sess.get_stats()
        return st["accepted"] / max(1, st["tested"])

    try:
        if not rate(lo) <= target <= rate(hi):
            raise ValueError(f"acceptance {target} is not reached between sigma = {lo} and {hi}")
        mid, r = hi, 1.0
        for _ in range(iters):
            mid = (lo * hi) ** 0.5
            r = rate(mid)
            if abs(r - target) <= tol:
                break
            lo, hi = (mid, hi) if r < target else (lo, mid)
        return mid, r
    finally:
        sess.close()


def measure(inputs, reps):
    import torch
    c = inputs.cfg
    sess = session_for(inputs)
    sess.prefill(inputs.context, c.n_ctx, c.horizon)
    for _ in range(2):
        _decode_spec(sess)
    rounds = _decode_spec(sess)
    st = sess.get_stats()
    t_spec = _time(torch, lambda: _decode_spec(sess), reps)
    _decode_target(sess, c.T)
    t_base = _time(torch, lambda: _decode_target(sess, c.T), reps)
    nothing = lambda: None
    t_draft = _phase(torch, sess, sess.draft_propose, nothing)
    t_verify = _phase(torch, sess, sess.target_verify, sess.draft_propose)
    t_accept = _phase(torch, sess, sess.accept_commit, lambda: (sess.draft_propose(), sess.target_verify()))
    t_step = _phase(torch, sess, sess.target_step, nothing)
    sess.close()
    return dict(t_spec=t_spec * 1e3, t_base=t_base * 1e3, rounds=rounds, tested=st["tested"], accepted=st["accepted"],
                committed=st["committed"], series_rounds=st["rounds"], draft=t_draft, verify=t_verify, accept=t_accept,
                step=t_step)


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg4")
    ap.add_argument("--K", type=int, nargs="*", default=None)
    ap.add_argument("--sigma", type=float, nargs="*", default=None)
    ap.add_argument("--calibrate", type=float, nargs="*", default=None, metavar="ALPHA",
                    help="sweep the temperatures at which the measured acceptance hits these rates")
    ap.add_argument("--series", type=int, default=1, help="independent series draws to average over (B = 1 configs)")
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args(argv)
    base = synth.get_config(a.config)
    if a.calibrate:
        a.sigma = []
        for t in a.calibrate:
            sigma, r = calibrate_sigma(synth.Inputs(a.config), t)
            print(f"acceptance {t:g}: sigma = {sigma:.4f} (measured {r:.3f})")
            a.sigma.append(sigma)
        print()
    points = [(K, base.sigma) for K in a.K] if a.K else [(base.K, s) for s in (a.sigma or [base.sigma])]
    print(f"| K | sigma | accept | L/round | E[L] Eq.7 | draft ms | verify ms | step ms | c | v | S Eq.8 | S patch-rate | "
          f"S batch | next K pays | spec ms | target-only ms |")
    print("|" + "---|" * 16)
    for K, sigma in points:
        acc = None
        for i in range(a.series):
            inputs = synth.Inputs(a.config, K=K, sigma=sigma, series_seed=base.series_seed + 100 * i)
            m = measure(inputs, a.reps)
            acc = m if acc is None else {k: acc[k] + m[k] for k in m}
        n = a.series
        alpha = acc["accepted"] / max(1, acc["tested"])
        L = acc["committed"] / max(1, acc["series_rounds"])
        draft, verify, accept, step = (acc[k] / n for k in ("draft", "verify", "accept", "step"))
        c, v = draft / K / step, (verify + accept) / step
        print(f"| {K} | {sigma:.4g} | {alpha:.3f} | {L:.2f} | {law.mean_block_length(alpha, K):.2f} | {draft:.3f} | {verify:.3f} | "
              f"{step:.3f} | {c:.3f} | {v:.3f} | {law.speedup(alpha, K, c, v):.2f} | {L * step / (draft + verify + accept):.2f} | "
              f"{acc['t_base'] / acc['t_spec']:.2f} | {'yes' if law.one_more_position_pays(alpha, K, c, v) else 'no'} | "
              f"{acc['t_spec'] / n:.2f} | {acc['t_base'] / n:.2f} |", flush=True)


if __name__ == "__main__":
    sys.exit(main())
