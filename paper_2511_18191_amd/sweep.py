"""Block-size and temperature sweeps on one GPU, reported next to the paper's throughput law.

    python -m paper_2511_18191_amd.sweep --config cfg4 --K 1 2 3 4 5 6 7 8 --series 8
    python -m paper_2511_18191_amd.sweep --config cfg2 --sigma 0.5 1 2

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
    rounds = 0
    while True:
        sess.round()
        rounds += 1
        if sess.num_active() == 0:
            return rounds


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
    ap.add_argument("--series", type=int, default=1, help="independent series draws to average over (B = 1 configs)")
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args(argv)
    base = synth.get_config(a.config)
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
        print(f"| {K} | {sigma:g} | {alpha:.3f} | {L:.2f} | {law.mean_block_length(alpha, K):.2f} | {draft:.3f} | {verify:.3f} | "
              f"{step:.3f} | {c:.3f} | {v:.3f} | {law.speedup(alpha, K, c, v):.2f} | {L * step / (draft + verify + accept):.2f} | "
              f"{acc['t_base'] / acc['t_spec']:.2f} | {'yes' if law.one_more_position_pays(alpha, K, c, v) else 'no'} | "
              f"{acc['t_spec'] / n:.2f} | {acc['t_base'] / n:.2f} |", flush=True)


if __name__ == "__main__":
    sys.exit(main())
