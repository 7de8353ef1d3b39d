"""Random-initialised transformer weights in a fixed, documented tensor order.

Order of one model's tensors (all float32, row-major, shapes as used in y = x @ W):
    W_e [P, D]
    per layer l = 0..L-1:
        g1 [D]  W_q [D, D]  W_k [D, D]  W_v [D, D]  W_o [D, D]  g2 [D]
        dense FFN:  W_1 [D, F]  W_2 [F, D]
        routed FFN: W_r [D, E], then per expert e: W_1[e] [D, F], W_2[e] [F, D]
    g_f [D]  W_h [D, P]
Matrices are i.i.d. N(0, std^2); RMSNorm gains are 1 unless `random_gains` is set (tests use
that to exercise the gain path).  For bf16 runs every tensor is rounded to the nearest bf16
value (ties to even) before anyone reads it, so both implementations start from equal inputs.
"""
import numpy as np


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16-representable float32 (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def weight_spec(m, patch):
    """List of (name, shape) in blob order for model config `m` and patch length `patch`."""
    D, F = m.d_model, m.d_ff
    spec = [("W_e", (patch, D))]
    for l in range(m.n_layers):
        spec += [(f"l{l}.g1", (D,)), (f"l{l}.W_q", (D, D)), (f"l{l}.W_k", (D, D)), (f"l{l}.W_v", (D, D)),
                 (f"l{l}.W_o", (D, D)), (f"l{l}.g2", (D,))]
        if m.n_experts > 0:
            spec.append((f"l{l}.W_r", (D, m.n_experts)))
            for e in range(m.n_experts):
                spec += [(f"l{l}.e{e}.W_1", (D, F)), (f"l{l}.e{e}.W_2", (F, D))]
        else:
            spec += [(f"l{l}.W_1", (D, F)), (f"l{l}.W_2", (F, D))]
    spec += [("g_f", (D,)), ("W_h", (D, patch))]
    return spec


def make_weights(m, patch, rng, dtype="fp32", std=0.02, random_gains=False):
    """Dict name -> float32 array, drawn in blob order from `rng` (a numpy Generator)."""
    out = {}
    for name, shape in weight_spec(m, patch):
        if len(shape) == 1:
            w = (1.0 + 0.2 * rng.standard_normal(shape)) if random_gains else np.ones(shape)
        else:
            w = std * rng.standard_normal(shape)
        w = w.astype(np.float32)
        out[name] = round_to_bf16(w) if dtype == "bf16" else w
    return out


def flatten_weights(m, patch, weights):
    """Concatenate the tensors in blob order into one float32 vector."""
    return np.concatenate([np.asarray(weights[n], dtype=np.float32).reshape(-1) for n, _ in weight_spec(m, patch)])
