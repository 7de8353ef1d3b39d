"""Block-size planner (Proposition "Marginal-gain condition for K", Remark "Estimating (alpha, c)",
Theorem "Hoeffding concentration"): estimate the acceptance rate from a few calibration rounds,
measure the cost ratios on the GPU, and choose K.

    python -m paper_2511_18191_amd.planner --config cfg4 --k-max 8 --validate
    python -m paper_2511_18191_amd.planner --config cfg2 --k-max 8 --validate

Steps, all on one handle created with K = k_max (`tsd_set_block_size` moves K below that):
  1. calibration: `rounds` speculative rounds at K = k_probe from the post-prefill state; the
     plug-in estimate is accepted / tested, its Hoeffding half-width uses the number of series
     (each series' accepted fraction is one independent [0, 1]-valued term);
  2. cost table: HIP-event times of one draft proposal, one verification + acceptance and one
     target-only step for every K in 1..k_max -> c(K) = draft / (K step), v(K) = (verify + accept) / step;
  3. the paper's rule with the pair (alpha, c, v) measured at k_probe, and the same maximisation of
     Eq. 8 with the measured c(K), v(K) (here verification is K + 1 tokens against a KV cache, so v
     grows with K once the batch fills the GPU);
  4. --validate: time whole decodes at every K and show where the measured optimum lies;
  5. the lock-step model of the whole batch (batch_decode_model): the block size with the shortest predicted decode,
     which, unlike Eq. 8, pays for the rounds in which only the slowest series are still decoding.
"""
import argparse
import sys

import numpy as np

import synth

from . import law
from .binding import session_for
from .sweep import _decode_spec, _decode_target, _phase, _time


def calibrate(sess, k_probe, rounds):
    """Acceptance estimate from `rounds` rounds at K = k_probe, starting at the post-prefill state."""
    sess.set_block_size(k_probe)
    sess.reset_decode()
    for _ in range(rounds):
        if sess.num_active() == 0:
            break
        sess.round()
    st = sess.get_series_stats().cpu().numpy()
    tested, accepted = st[:, 1], st[:, 2]
    seen = tested > 0
    per_series = accepted[seen] / tested[seen]
    n = int(seen.sum())
    return dict(alpha=float(accepted.sum() / max(1, tested.sum())), alpha_mean_of_series=float(per_series.mean()) if n else 0.0,
                n_histories=n, halfwidth=law.acceptance_confidence(max(1, n)))


def cost_table(sess, k_max, reps=10):
    import torch
    nothing = lambda: None
    out = {}
    for K in range(1, k_max + 1):
        sess.set_block_size(K)
        draft = _phase(torch, sess, sess.draft_propose, nothing, reps)
        verify = _phase(torch, sess, sess.target_verify, sess.draft_propose, reps)
        accept = _phase(torch, sess, sess.accept_commit, lambda: (sess.draft_propose(), sess.target_verify()), reps)
        step = _phase(torch, sess, sess.target_step, nothing, reps)
        out[K] = dict(draft=draft, verify=verify, accept=accept, step=step, c=draft / K / step, v=(verify + accept) / step)
    return out


def plan(alpha, costs, k_probe):
    """K by the paper's rule (constant c, v measured at k_probe) and by Eq. 8 over the measured table."""
    k_max = max(costs)
    c0, v0 = costs[k_probe]["c"], costs[k_probe]["v"]
    k_rule = law.best_block_size(alpha, c0, v0, k_max=k_max)
    S = {K: law.mean_block_length(alpha, K) / (costs[K]["c"] * K + costs[K]["v"]) for K in costs}
    return dict(k_rule=k_rule, k_table=max(S, key=S.get), S_table=S, S_rule={K: law.speedup(alpha, K, c0, v0) for K in costs})


def round_times(sess, context, n_ctx, horizon, K, reps=4):
    """Wall time of one round (graph replay and the delivery of the count) from the post-prefill state of a batch of n
    series, for n at the size classes of the active list (32, 24, 16, 12, 8, 4, 2, 1 thirty-seconds of the batch), at K
    positions and at one.  Returns {(n, k): seconds}.  Leaves the handle prefilled with the whole batch at block size K."""
    import time
    import torch
    B = context.shape[0]
    sizes = sorted({max(1, (B * f + 31) // 32) for f in (32, 24, 16, 12, 8, 4, 2, 1)}, reverse=True)
    cost = {}
    for n in sizes:
        sess.prefill(context[:n], n_ctx, horizon)
        for k in sorted({K, 1}):
            sess.set_block_size(k)
            ts = []
            for _ in range(reps):
                sess.reset_decode()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                sess.round()
                sess.num_active()
                torch.cuda.synchronize()
                ts.append(time.perf_counter() - t0)
            cost[(n, k)] = min(ts[1:])
        sess.set_block_size(K)
    sess.prefill(context, n_ctx, horizon)
    return cost


def batch_decode_model(tested, accepted, cost, K, T, reps=100):
    """Decode time of a whole batch as the capped-geometric law predicts it once the lock-step is modelled
    (law.simulate_batch_rounds: every series draws its blocks, the batch runs until its slowest series has its T
    patches), each simulated round priced with `cost` (round_times: linear in the active count between the measured
    sizes and in the positions between one and K).  tested, accepted: per-series counters of a decode.  Two acceptance
    models bracket a real batch: every series at the pooled measured rate (the law's i.i.d. assumption), and every series
    at its own accepted / tested (which adds the sampling noise of a dozen tests per series to the real spread).
    Also the block size K' <= K with the shortest predicted decode (mean of the two models)."""
    tested, accepted = np.asarray(tested, dtype=np.float64), np.asarray(accepted, dtype=np.float64)
    B = tested.shape[0]
    pooled = float(accepted.sum() / max(1.0, tested.sum()))
    raw = np.where(tested > 0, accepted / np.maximum(tested, 1.0), pooled)
    sizes = sorted({n for n, _ in cost})
    ns = np.array(sizes, dtype=np.float64)
    hi_t, lo_t = np.array([cost[(n, K)] for n in sizes]), np.array([cost[(n, 1)] for n in sizes])

    def price(n, k):
        hi = np.interp(n, ns, hi_t)
        if K == 1:
            return hi
        lo = np.interp(n, ns, lo_t)
        return lo + (hi - lo) * (k - 1) / (K - 1)

    def predict(alpha_b, k_block, n_rep):
        act, pos = law.simulate_batch_rounds(alpha_b, k_block, T, reps=n_rep, seed=0)
        on = act > 0
        t = np.where(on, price(act.astype(np.float64), pos.astype(np.float64)), 0.0).sum(axis=1)
        return float(on.sum(axis=1).mean()), float(t.mean())
    out = {"model": "capped-geometric blocks per series, the batch runs until its slowest series is done (Monte Carlo); rounds priced "
                    "with measured round times by active count and positions; acceptance either pooled (i.i.d.) or per series",
           "round_ms_by_active": {str(n): round(cost[(n, K)] * 1e3, 4) for n in reversed(sizes)},
           "round_ms_by_active_at_one_position": {str(n): round(cost[(n, 1)] * 1e3, 4) for n in reversed(sizes)},
           "acceptance_spread_5_50_95": [float(np.quantile(raw, q)) for q in (0.05, 0.5, 0.95)]}
    for name, alpha_b in (("pooled_acceptance", np.full(B, pooled)), ("per_series_acceptance", raw)):
        r, t = predict(alpha_b, K, reps)
        out[name] = {"predicted_rounds": r, "predicted_ms": t * 1e3}
    by_k = {k: 0.5 * (predict(np.full(B, pooled), k, 40)[1] + predict(raw, k, 40)[1]) for k in range(1, K + 1)}
    out["predicted_ms_by_block_size"] = {str(k): round(v * 1e3, 3) for k, v in by_k.items()}
    out["best_block_size"] = min(by_k, key=by_k.get)
    return out


def main(argv=None):
    import torch
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg4")
    ap.add_argument("--k-max", type=int, default=8)
    ap.add_argument("--k-probe", type=int, default=2)
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--series", type=int, default=None, help="batch size of the calibration / decode batch")
    ap.add_argument("--validate", action="store_true")
    a = ap.parse_args(argv)
    inputs = synth.Inputs(a.config, K=a.k_max, B=a.series)
    c = inputs.cfg
    sess = session_for(inputs)
    sess.prefill(inputs.context, c.n_ctx, c.horizon)
    cal = calibrate(sess, a.k_probe, a.rounds)
    costs = cost_table(sess, a.k_max)
    p = plan(cal["alpha"], costs, a.k_probe)
    lo, hi = max(0.0, cal["alpha"] - cal["halfwidth"]), min(1.0, cal["alpha"] + cal["halfwidth"])
    p_lo, p_hi = plan(lo, costs, a.k_probe), plan(hi, costs, a.k_probe)
    print(f"{c.name}: B={c.batch} sigma={c.sigma:g}; calibration {a.rounds} rounds at K={a.k_probe}: acceptance "
          f"{cal['alpha']:.3f} (mean of per-series fractions {cal['alpha_mean_of_series']:.3f}, {cal['n_histories']} series, "
          f"95 % Hoeffding half-width {cal['halfwidth']:.3f})")
    print(f"paper's rule with (c, v) at K={a.k_probe}: K* = {p['k_rule']} (interval ends: {p_lo['k_rule']} .. {p_hi['k_rule']}); "
          f"Eq. 8 over the measured cost table: K* = {p['k_table']} (interval ends: {p_lo['k_table']} .. {p_hi['k_table']})\n")
    hdr = "| K | draft ms | verify+accept ms | step ms | c(K) | v(K) | S Eq.8, c,v fixed | S Eq.8, measured c(K),v(K) |"
    if a.validate:
        hdr += " acceptance | patches/round | spec ms | target-only ms | S batch | S patch-rate |"
    print(hdr)
    print("|" + "---|" * (hdr.count("|") - 1))
    for K in range(1, a.k_max + 1):
        t = costs[K]
        row = (f"| {K} | {t['draft']:.3f} | {t['verify'] + t['accept']:.3f} | {t['step']:.3f} | {t['c']:.3f} | {t['v']:.3f} | "
               f"{p['S_rule'][K]:.2f} | {p['S_table'][K]:.2f} |")
        if a.validate:
            sess.set_block_size(K)
            _decode_spec(sess)
            st = sess.get_stats()
            t_spec = _time(torch, lambda: _decode_spec(sess), 3)
            t_base = _time(torch, lambda: _decode_target(sess, c.T), 3)
            L = st["committed"] / max(1, st["rounds"])
            row += (f" {st['accepted'] / max(1, st['tested']):.3f} | {L:.2f} | {t_spec * 1e3:.2f} | {t_base * 1e3:.2f} | "
                    f"{t_base / t_spec:.2f} | {L * t['step'] / (t['draft'] + t['verify'] + t['accept']):.2f} |")
        print(row, flush=True)
    if c.batch > 1:
        sess.set_block_size(a.k_max)
        _decode_spec(sess)
        per = sess.get_series_stats().cpu().numpy()
        m = batch_decode_model(per[:, 1], per[:, 2], round_times(sess, inputs.context, c.n_ctx, c.horizon, a.k_max), a.k_max, c.T)
        print(f"\nlock-step model of the whole batch (capped-geometric blocks per series until the slowest is done, measured round "
              f"times by active count): predicted decode ms by block size {m['predicted_ms_by_block_size']}; shortest at K = {m['best_block_size']}")
    sess.close()


if __name__ == "__main__":
    sys.exit(main())
