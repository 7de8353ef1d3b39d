"""Per-stage times of the one-launch draft phase (the library's tsd_trace_draft tap).

    python -m paper_2511_18191_amd.trace_draft --config cfg2

One workgroup notes the 100 MHz wall clock after each of its stage barriers; the table gives the
median over --reps traced launches of every stage's duration, per draft step and layer.
"""
import argparse
import sys

import numpy as np

import synth

from .binding import TSD_FLAG_FUSED_DRAFT, session_for


def stage_names(steps, layers):
    names = ["set-up: series, zeroed rows", "set-up: page tables, lengths, step 1 inputs"]
    for s in range(1, steps + 1):
        names += [f"step {s}: positions, rotary factors", f"step {s}: patch embedding"]
        for l in range(layers):
            names += [f"step {s} layer {l}: {x}" for x in ("QKV + RoPE + cache write", "attention", "attention output", "FFN up + GELU", "FFN down")]
        names.append(f"step {s}: head")
    return names


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--reps", type=int, default=9)
    a = ap.parse_args(argv)
    inputs = synth.Inputs(a.config, B=a.batch)
    c = inputs.cfg
    sess = session_for(inputs, flags=TSD_FLAG_FUSED_DRAFT)
    sess.prefill(inputs.context, c.n_ctx, c.horizon)
    runs = []
    for _ in range(a.reps):
        t = np.asarray(sess.trace_draft(), dtype=np.int64)
        runs.append(np.diff(t) * 0.01)          # microseconds per stage (the first stamp is the origin)
    d = np.median(np.stack(runs), axis=0)
    names = stage_names(c.K, c.draft.n_layers)[1:]
    assert len(names) == len(d), (len(names), len(d))
    print(f"{c.name}: B={c.batch} K={c.K} draft {c.draft.n_layers}L/d{c.draft.d_model}; workgroup 0, median of {a.reps} launches, "
          f"whole phase {d.sum():.1f} us after the first barrier\n")
    print("| stage | us |")
    print("|---|---|")
    for n, v in zip(names, d):
        print(f"| {n} | {v:.2f} |")
    per_step = d[1:].reshape(c.K, -1)
    print(f"\nper step: " + ", ".join(f"{x:.1f}" for x in per_step.sum(axis=1)) + " us")


if __name__ == "__main__":
    sys.exit(main())
