"""Host arithmetic of the paper's throughput law: reporting next to measured numbers, and the planner.

Eq. 7: under a per-position acceptance rate alpha the committed patches per round follow a capped
geometric law with mean E[L] = (1 - alpha^(K+1)) / (1 - alpha).  Eq. 8: with c the draft-to-target
cost ratio per call and v the verification-to-forward cost ratio, one round is worth
S(K) = E[L] / (c K + v) target-only steps.  Marginal criterion: K + 1 beats K exactly when
alpha^(K+1) (c K + v) >= c E[L_K].
"""


def mean_block_length(alpha, K):
    if alpha >= 1.0:
        return float(K + 1)
    return (1.0 - alpha ** (K + 1)) / (1.0 - alpha)


def speedup(alpha, K, c, v):
    return mean_block_length(alpha, K) / (c * K + v)


def one_more_position_pays(alpha, K, c, v):
    return alpha ** (K + 1) * (c * K + v) >= c * mean_block_length(alpha, K)


def best_block_size(alpha, c, v, k_max=16):
    """Largest K (from 1) up to which every added position paid, per the marginal criterion."""
    K = 1
    while K < k_max and one_more_position_pays(alpha, K, c, v):
        K += 1
    return K


def acceptance_confidence(n_histories, delta=0.05):
    """Half-width eps of the two-sided interval around the plug-in acceptance estimate from
    n independent histories (Theorem "Hoeffding concentration"): 2 exp(-2 n eps^2) = delta."""
    import math
    return math.sqrt(math.log(2.0 / delta) / (2.0 * n_histories))


def simulate_batch_rounds(alpha_b, K, T, reps=200, seed=0):
    """Monte Carlo of the capped-geometric law (Eq. 7) for a whole batch that decodes in lock-step rounds: series b
    accepts each tested position independently with probability alpha_b[b], a round tests min(K, patches it still
    needs) positions and commits the leading accepts plus one (cut at the horizon), and the batch runs until its
    slowest series has its T patches (the per-example stalls that desynchronise a batch, Sec. "Limitations").
    Returns (active, positions): int arrays [reps, R] with the series still decoding before each round and the
    positions the round's passes run (min(K, most patches any series still needs)); zero once a repetition is done."""
    import numpy as np
    rng = np.random.default_rng(seed)
    a = np.clip(np.asarray(alpha_b, dtype=np.float64), 0.0, 1.0)[None, :]
    B = a.shape[1]
    left = np.full((reps, B), int(T), dtype=np.int64)
    active, positions = [], []
    while (left > 0).any():
        on = left > 0
        active.append(on.sum(axis=1))
        positions.append(np.minimum(K, left.max(axis=1)))
        kb = np.minimum(K, left)                                              # positions each series tests
        ok = rng.random((reps, B, K)) < a[:, :, None]
        lead = np.cumprod(ok, axis=2).sum(axis=2)                             # leading accepts among K draws
        n = np.minimum(lead, kb)
        left = np.where(on, left - np.minimum(n + 1, left), left)
    return np.stack(active, axis=1), np.stack(positions, axis=1)
