"""Continuous batching over the slots of one handle: a stream of series is forecast through B
slots, and a slot is handed to the next waiting series as soon as its forecast is complete
(`tsd_refill`), instead of idling until the slowest series of its batch has finished.

    python -m paper_2511_18191_amd.serve --config cfg2 --batches 4

prints, for S = batches x B series, the time of batch-synchronous processing (prefill + decode of
one batch after the other) and of the continuous stream, both including the context prefill.
"""
import argparse
import sys
import time

import numpy as np

import synth

from .binding import session_for


def run_stream(sess, contexts, n_ctx, horizon, track=False):
    """Forecast every row of `contexts` ([S, n_ctx * P] raw steps, S >= 1) through the slots of
    `sess`.  Returns (forecasts [S, horizon] on the GPU, placement): placement[s] = (slot, the slot's
    round counter when series s started) if track, else None."""
    torch = sess.torch
    S = contexts.shape[0]
    B = min(sess.cfg.max_batch, S)
    P = sess.cfg.patch
    T = -(-horizon // P)
    ctx_dev = sess._to_dev(contexts, torch.float32)
    out = torch.empty(S, horizon, dtype=torch.float32, device=sess.device)
    sess.prefill(ctx_dev[:B], n_ctx, horizon)
    owner = list(range(B))              # series in each slot, -1 once harvested and not replaced
    placement = [None] * S
    if track:
        for s in range(B):
            placement[s] = (s, 0)
    nxt, pending = B, B
    live = B                            # slots that were decoding after the last look
    while pending:
        sess.round()
        n = sess.num_active()
        if n == live:                   # nobody finished in this round: nothing to harvest
            continue
        committed = sess.get_state()["committed"].cpu().numpy()
        done = [b for b in range(B) if owner[b] >= 0 and committed[b] >= T]
        if not done:
            continue
        fc = sess.get_forecast()
        with torch.cuda.stream(sess.stream):
            out[[owner[b] for b in done]] = fc[done]
        sess.sync()
        pending -= len(done)
        take = min(len(done), S - nxt)
        if take:
            slots = done[:take]
            if track:
                rounds = sess.get_series_stats()[:, 0].cpu().numpy()
                for j, b in enumerate(slots):
                    placement[nxt + j] = (b, int(rounds[b]))
            sess.refill(slots, ctx_dev[nxt:nxt + take])
            for j, b in enumerate(slots):
                owner[b] = nxt + j
            nxt += take
            pending += take
            n = sess.num_active()
        for b in done[take:]:
            owner[b] = -1
        live = n
    return out, placement


def run_batches(sess, contexts, n_ctx, horizon):
    """The same stream, one batch after the other (each batch waits for its slowest series)."""
    torch = sess.torch
    S, B = contexts.shape[0], sess.cfg.max_batch
    ctx_dev = sess._to_dev(contexts, torch.float32)
    out = torch.empty(S, horizon, dtype=torch.float32, device=sess.device)
    for s0 in range(0, S, B):
        sess.prefill(ctx_dev[s0:s0 + B], n_ctx, horizon)
        sess.run_rounds()
        fc = sess.get_forecast()
        with torch.cuda.stream(sess.stream):
            out[s0:s0 + B] = fc
        sess.sync()
    return out


def main(argv=None):
    import torch
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--batches", type=int, default=4)
    ap.add_argument("--sigma", type=float, default=None)
    ap.add_argument("--K", type=int, default=None)
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args(argv)
    base = synth.get_config(a.config)
    inputs = synth.Inputs(a.config, B=base.batch * a.batches, sigma=a.sigma, K=a.K)
    c = inputs.cfg
    sess = session_for(inputs, max_batch=base.batch)
    res = {}
    for name, fn in (("batch-synchronous", run_batches), ("continuous (refill)", lambda *x: run_stream(*x)[0])):
        fn(sess, inputs.context, c.n_ctx, c.horizon)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.reps):
            out = fn(sess, inputs.context, c.n_ctx, c.horizon)
        torch.cuda.synchronize()
        res[name] = ((time.perf_counter() - t0) / a.reps, out)
    S = c.batch
    print(f"{c.name}: {S} series through {base.batch} slots, K={c.K} sigma={c.sigma:g} H={c.horizon} (prefill of the context included)\n")
    print("| mode | ms for the stream | series/s | forecast steps/s |")
    print("|---|---|---|---|")
    for name, (t, _) in res.items():
        print(f"| {name} | {t * 1e3:.2f} | {S / t:.0f} | {S * c.horizon / t:.3e} |")
    a_, b_ = res["batch-synchronous"][1], res["continuous (refill)"][1]
    print(f"\nspeedup of the continuous stream: {res['batch-synchronous'][0] / res['continuous (refill)'][0]:.2f}x; "
          f"both forecasts finite: {bool(torch.isfinite(a_).all() and torch.isfinite(b_).all())}")
    sess.close()


if __name__ == "__main__":
    sys.exit(main())
