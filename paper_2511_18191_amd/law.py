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
