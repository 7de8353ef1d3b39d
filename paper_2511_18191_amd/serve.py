"""Continuous batching over the slots of one handle: a stream of series is forecast through B
slots, and a slot is handed to the next waiting series as soon as its forecast is complete
(`tsd_refill`), instead of idling until the slowest series of its batch has finished.

    python -m paper_2511_18191_amd.serve --config cfg2 --batches 4

prints, for S = batches x B series, the time of the target-only loop and of speculative decoding batch after
batch (prefill + decode of one batch after the other) and of the continuous stream, all including the context
prefill, and the same with the prefill time taken off (the part speculation can speed up).
"""
import argparse
import sys
import time

import numpy as np

import synth

from .binding import session_for


def run_stream(sess, contexts, n_ctx, horizon, track=False, min_refill=1):
    """Forecast every row of `contexts` ([S, n_ctx * P] raw steps, S >= 1) through the slots of
    `sess`.  A freed slot waits until `min_refill` slots are free (or nothing is decoding any more), so that
    the prefill pass of the newcomers, which costs a launch-bound pass however few they are, is shared.
    Returns (forecasts [S, horizon] on the GPU, placement): placement[s] = (slot, the slot's
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
    free = []                           # harvested slots waiting for a newcomer
    while pending:
        sess.round()
        n = sess.num_active()
        if n == live:                   # nobody finished in this round: nothing to harvest
            continue
        committed = sess.get_state()["committed"].cpu().numpy()
        done = [b for b in range(B) if owner[b] >= 0 and committed[b] >= T]
        if done:
            fc = sess.get_forecast()
            with torch.cuda.stream(sess.stream):
                out[[owner[b] for b in done]] = fc[done]
            sess.sync()
            pending -= len(done)
            for b in done:
                owner[b] = -1
            free += done
        take = min(len(free), S - nxt)
        if take and (len(free) >= min_refill or n == 0 or S - nxt <= len(free)):
            slots, free = free[:take], free[take:]
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
        live = n
    return out, placement


def run_batches(sess, contexts, n_ctx, horizon, target_only=False):
    """The same stream, one batch after the other (each batch waits for its slowest series); target_only: the
    target-only autoregressive loop (Eq. 1) instead of speculative rounds."""
    torch = sess.torch
    S, B = contexts.shape[0], sess.cfg.max_batch
    P = sess.cfg.patch
    T = -(-horizon // P)
    ctx_dev = sess._to_dev(contexts, torch.float32)
    out = torch.empty(S, horizon, dtype=torch.float32, device=sess.device)
    for s0 in range(0, S, B):
        sess.prefill(ctx_dev[s0:s0 + B], n_ctx, horizon)
        if target_only:
            for _ in range(T):
                sess.target_step()
        else:
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
    ap.add_argument("--min-refill", type=int, nargs="+", default=None,
                    help="free slots to wait for before a refill (default: 1 and a quarter of the slots)")
    a = ap.parse_args(argv)
    base = synth.get_config(a.config)
    inputs = synth.Inputs(a.config, B=base.batch * a.batches, sigma=a.sigma, K=a.K)
    c = inputs.cfg
    sess = session_for(inputs, max_batch=base.batch)
    modes = [("target-only, batch after batch", lambda *x: run_batches(*x, target_only=True)),
             ("speculative, batch after batch", run_batches)]
    for m in (a.min_refill or [1, max(1, base.batch // 4)]):
        modes.append((f"speculative, continuous (refill once {m} slot{'s are' if m > 1 else ' is'} free)",
                      lambda *x, m=m: run_stream(*x, min_refill=m)[0]))
    res = {}
    for name, fn in modes:
        fn(sess, inputs.context, c.n_ctx, c.horizon)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.reps):
            out = fn(sess, inputs.context, c.n_ctx, c.horizon)
        torch.cuda.synchronize()
        res[name] = ((time.perf_counter() - t0) / a.reps, out)
    S = c.batch
    t_prefill = 0.0
    for _ in range(a.reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sess.prefill(inputs.context[:base.batch], c.n_ctx, c.horizon)
        torch.cuda.synchronize()
        t_prefill += (time.perf_counter() - t0) / a.reps
    print(f"{c.name}: {S} series through {base.batch} slots, K={c.K} sigma={c.sigma:g} H={c.horizon} (prefill of the context included: "
          f"{t_prefill * 1e3:.2f} ms per batch of {base.batch})\n")
    print("| mode | ms for the stream | series/s | forecast steps/s | vs target-only | decode part only vs target-only |")
    print("|---|---|---|---|---|---|")
    t_base = res["target-only, batch after batch"][0]
    pf = t_prefill * a.batches
    for name, (t, _) in res.items():
        print(f"| {name} | {t * 1e3:.2f} | {S / t:.0f} | {S * c.horizon / t:.3e} | {t_base / t:.2f}x | {(t_base - pf) / max(t - pf, 1e-9):.2f}x |")
    fin = all(bool(torch.isfinite(o).all()) for _, o in res.values())
    print(f"\n(decode part: the stream's time less {a.batches} batch prefills; all forecasts finite: {fin})")
    sess.close()


if __name__ == "__main__":
    sys.exit(main())
