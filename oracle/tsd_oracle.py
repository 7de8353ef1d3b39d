"""CPU oracle for Gaussian speculative decoding of patch-autoregressive forecasters.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the GPU library
must compute.  Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does, and this module imports nothing from the product.

Everything is float64 numpy, one series at a time, with NO KV cache: every model evaluation is
a full causal forward over the whole current history, so the "one pass equals K+1 passes"
property (Sec. "Single-Pass Verification") is something the tests can check rather than assume.

What the paper fixes and what it leaves open
  * fixed by the paper: the patch-autoregressive loop (Eq. 1), Gaussian surrogate heads
    (Eq. 4), the 1/d-scaled log-ratio statistic (Eq. 5) and its mean-propagating special case
    (Eq. 6), target-mean fallback, bonus patch on full acceptance, single causal verification
    pass, normalisation frozen on the context, and the order of steps of one round
    (Algorithm "One speculative round").
  * open in the paper, fixed here (same choices as the GPU library's header documents):
    the transformer's internals (pre-norm RMSNorm eps 1e-6, half-split RoPE base 10000,
    tanh-GELU, no biases, softmax-router top-2 MoE with renormalised gates), instance
    normalisation (mean / population std with eps 1e-5 under the root), the uniform draw
    (Philox4x32-10 keyed by seed, counter = (series, round, position, 0), 23-bit mid-point
    lattice), "u <= alpha" evaluated as log u <= min(0, ell), the horizon: T = ceil(H / P)
    patches, a round of a series with r patches left proposes and tests min(K, r) positions
    (nothing is proposed for patches that could never be committed) and a bonus patch beyond T
    is dropped.

Pins (tests/test_oracle_*.py): Philox known-answer vectors; closed forms of Eq. 5 / Eq. 6 and
of the fidelity identity (Eq. 9); the model collapsing to a two-matmul closed form when the
mixing matrices are zero; causality; single pass == K+1 passes; brute force over accept
patterns; draft == target; sigma -> 0; the capped-geometric block-length law (Eq. 7); for the
sampled variants a Kolmogorov-Smirnov test of the normal draws, the equal-covariance closed form
2 Phi(-Delta/2) of the unscaled stochastic rule, a quadrature of the tempered rule's mean
acceptance, and the fallback-noise energy r^2; for the threshold rule its equivalence to the
ratio rule under the constant draw u = exp(-1/2) and a hand-built boundary case; for the
batch-synchronised loop the reduction to the unsynchronised one at batch 1 and on identical series,
and the per-round minimum recomputed from each series' own record.
The full transformer forward (several layers, heads and tokens) is pinned against a composition
of torch float64 library routines (rms_norm, scaled_dot_product_attention with its own causal mask,
tanh gelu) and a rotary embedding written a second way (complex multiplication, itself checked
against hand-written rotations).
"""
import math

import numpy as np

RMS_EPS = 1e-6      # inside the root of RMSNorm
NORM_EPS = 1e-5     # inside the root of the instance normalisation
ROPE_BASE = 10000.0

# ----------------------------------------------------------------------------------------------
# Counter-based uniforms: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11)
# ----------------------------------------------------------------------------------------------
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """Ten rounds of Philox-4x32 on python ints.  counter: 4 words, key: 2 words -> 4 words."""
    c0, c1, c2, c3 = (int(c) & _MASK32 for c in counter)
    k0, k1 = (int(k) & _MASK32 for k in key)
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        c0, c1, c2, c3 = (p1 >> 32) ^ c1 ^ k0, p1 & _MASK32, (p0 >> 32) ^ c3 ^ k1, p0 & _MASK32
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return c0, c1, c2, c3


def philox4x32_10_bulk(c0, c1, c2, c3, key, all_words=False):
    """Vectorised form of `philox4x32_10` over uint64 arrays of counters (word 0 only, or the four
    output words stacked on a new last axis with all_words=True)."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & np.uint64(_MASK32) for c in np.broadcast_arrays(c0, c1, c2, c3))
    k0, k1 = int(key[0]) & _MASK32, int(key[1]) & _MASK32
    m32 = np.uint64(_MASK32)
    s32 = np.uint64(32)
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M0) * c0
        p1 = np.uint64(_PHILOX_M1) * c2
        c0, c1, c2, c3 = (p1 >> s32) ^ c1 ^ np.uint64(k0), p1 & m32, (p0 >> s32) ^ c3 ^ np.uint64(k1), p0 & m32
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return np.stack([c0, c1, c2, c3], axis=-1) if all_words else c0


def word_to_uniform(w):
    """Top 23 bits of a 32-bit word, placed at cell mid-points: exact in fp32, strictly in (0, 1)."""
    return ((int(w) >> 9) + 0.5) * 2.0 ** -23


def uniform(seed, b, r, i):
    """The uniform of Algorithm "One speculative round" for series b, that series' round r
    (from 0) and proposal position i (1-based).  Key = (low, high) 32 bits of the seed."""
    w = philox4x32_10((b, r, i, 0), (seed & _MASK32, (seed >> 32) & _MASK32))
    return word_to_uniform(w[0])


# Standard normal draws for the sampled variants (Sec. "Fallback Correction and Sampled Variants").
# The paper only says "epsilon"; fixed here: element e of the patch drawn for (series b, round r,
# position i) in stream s comes from the Philox block with counter (b, r, i, s * 2^16 + e // 4);
# its four words give four lattice uniforms u0..u3 (as above) and two Box-Muller pairs
#   z0, z1 = sqrt(-2 ln u0) * (cos, sin)(2 pi u1),   z2, z3 = sqrt(-2 ln u2) * (cos, sin)(2 pi u3),
# and element e takes z_(e mod 4).  Stream 1 feeds proposals, stream 2 the fallback / bonus patch;
# the acceptance uniform keeps the fourth counter word 0, so the three never share a block.
STREAM_PROPOSAL = 1
STREAM_FALLBACK = 2


def _box_muller(words):
    """[..., 4] Philox words -> [..., 4] standard normals."""
    u = ((np.asarray(words, dtype=np.uint64) >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23
    rad0, rad1 = np.sqrt(-2.0 * np.log(u[..., 0])), np.sqrt(-2.0 * np.log(u[..., 2]))
    a0, a1 = 2.0 * np.pi * u[..., 1], 2.0 * np.pi * u[..., 3]
    return np.stack([rad0 * np.cos(a0), rad0 * np.sin(a0), rad1 * np.cos(a1), rad1 * np.sin(a1)], axis=-1)


def normal(seed, b, r, i, stream, P):
    """The P standard normal draws of series b, round r, position i (1-based), stream `stream`."""
    key = (seed & _MASK32, (seed >> 32) & _MASK32)
    blocks = [philox4x32_10((b, r, i, (stream << 16) + j), key) for j in range(-(-P // 4))]
    return _box_muller(np.array(blocks, dtype=np.uint64)).reshape(-1)[:P]


def normal_bulk(seed, b, r, i, stream, P):
    """`normal` over broadcastable integer arrays b, r, i: returns [..., P]."""
    key = (seed & _MASK32, (seed >> 32) & _MASK32)
    b, r, i = np.broadcast_arrays(np.asarray(b, dtype=np.uint64), np.asarray(r, dtype=np.uint64), np.asarray(i, dtype=np.uint64))
    j = np.arange(-(-P // 4), dtype=np.uint64) + np.uint64(stream << 16)
    w = philox4x32_10_bulk(b[..., None], r[..., None], i[..., None], j, key, all_words=True)   # [..., P/4, 4]
    z = _box_muller(w)
    return z.reshape(z.shape[:-2] + (-1,))[..., :P]


# ----------------------------------------------------------------------------------------------
# Model: decoder-only causal patch transformer with a point head (Sec. "Preliminaries", Eq. 1)
# ----------------------------------------------------------------------------------------------
def rmsnorm(x, g):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + RMS_EPS) * g


def gelu_tanh(z):
    return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))


def rope(x, pos):
    """Rotary embedding, half-split pairing.  x: [n, heads, hd]; pos: [n] absolute token index.
    Pair (i, i + hd/2) is rotated by the angle pos * base^(-2 i / hd)."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = ROPE_BASE ** (-2.0 * np.arange(half) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None, None] * inv_freq[None, None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax(z, axis=-1):
    z = z - np.max(z, axis=axis, keepdims=True)
    e = np.exp(z)
    return e / np.sum(e, axis=axis, keepdims=True)


def attention(q, k, v):
    """Causal multi-head attention.  q, k, v: [n, heads, hd] -> [n, heads * hd]."""
    n, H, hd = q.shape
    out = np.empty((n, H, hd))
    mask = np.tril(np.ones((n, n), dtype=bool))        # key index <= query index
    for h in range(H):
        s = q[:, h, :] @ k[:, h, :].T / math.sqrt(hd)
        s = np.where(mask, s, -np.inf)
        out[:, h, :] = softmax(s, axis=-1) @ v[:, h, :]
    return out.reshape(n, H * hd)


def ffn_dense(b, W, l):
    return gelu_tanh(b @ W[f"l{l}.W_1"]) @ W[f"l{l}.W_2"]


def ffn_routed(b, W, l, m, forced=None, info=None):
    """Softmax router over all experts, top-k by probability (ties -> lower index), the chosen
    probabilities renormalised to sum to one, no capacity limit.

    forced (comparison aid, default off): int array [n, top_k]; token t uses the experts forced[t]
    instead of its own top-k (a row of -1 leaves the token free), with this function's own
    probabilities renormalised over that set as gates.  The top-k choice is the one discrete step of
    the model: an implementation that rounds differently can pick another expert where two
    probabilities nearly tie, after which the two outputs are simply different functions; with the
    choice imposed, the rest can be compared at a floating-point tolerance.
    info, if a list, receives per token (own top-k tuple, log(p_k / p_(k+1)): the gap between the
    last expert taken and the first one left out, inf when top_k = n_experts)."""
    probs = softmax(b @ W[f"l{l}.W_r"], axis=-1)                   # [n, E]
    out = np.zeros_like(b)
    for t in range(b.shape[0]):
        ranked = sorted(range(m.n_experts), key=lambda e: (-probs[t, e], e))
        order = ranked[: m.top_k]
        if info is not None:
            gap = math.inf if m.top_k >= m.n_experts else math.log(probs[t, ranked[m.top_k - 1]] / probs[t, ranked[m.top_k]])
            info.append((tuple(order), gap))
        if forced is not None and forced[t][0] >= 0:
            order = [int(e) for e in forced[t]]
        z = sum(probs[t, e] for e in order)
        for e in order:
            y = gelu_tanh(b[t] @ W[f"l{l}.e{e}.W_1"]) @ W[f"l{l}.e{e}.W_2"]
            out[t] += (probs[t, e] / z) * y
    return out


def forward(W, m, tokens, forced_experts=None, route_info=None):
    """Full causal forward.  tokens: [n, P] normalised patches at positions 0..n-1.
    Returns mu: [n, P]; row j is the predicted mean of patch j + 1 given patches 0..j.
    forced_experts [layers, >= n, top_k] / route_info (a list that receives one list per layer): see
    `ffn_routed`; routed models only, comparison aid."""
    tokens = np.asarray(tokens, dtype=np.float64)
    n = tokens.shape[0]
    H, hd = m.n_heads, m.d_model // m.n_heads
    pos = np.arange(n)
    x = tokens @ W["W_e"]
    for l in range(m.n_layers):
        a = rmsnorm(x, W[f"l{l}.g1"])
        q = rope((a @ W[f"l{l}.W_q"]).reshape(n, H, hd), pos)
        k = rope((a @ W[f"l{l}.W_k"]).reshape(n, H, hd), pos)
        v = (a @ W[f"l{l}.W_v"]).reshape(n, H, hd)
        x = x + attention(q, k, v) @ W[f"l{l}.W_o"]
        b = rmsnorm(x, W[f"l{l}.g2"])
        if m.n_experts > 0:
            inf_l = [] if route_info is not None else None
            x = x + ffn_routed(b, W, l, m, None if forced_experts is None else forced_experts[l][:n], inf_l)
            if route_info is not None:
                route_info.append(inf_l)
        else:
            x = x + ffn_dense(b, W, l)
    return rmsnorm(x, W["g_f"]) @ W["W_h"]


def as_f64(weights):
    return {k: np.asarray(v, dtype=np.float64) for k, v in weights.items()}


# ----------------------------------------------------------------------------------------------
# Frozen instance normalisation (Sec. "Single-Pass Verification": statistics from the context only)
# ----------------------------------------------------------------------------------------------
def context_stats(context):
    context = np.asarray(context, dtype=np.float64)
    m = context.mean()
    s = math.sqrt(context.var() + NORM_EPS)
    return m, s


# ----------------------------------------------------------------------------------------------
# Acceptance statistic (Eq. 5) and one round (Algorithm "One speculative round")
# ----------------------------------------------------------------------------------------------
def energy(u):
    """Per-dimension energy ||u||_d^2 = ||u||_2^2 / d."""
    u = np.asarray(u, dtype=np.float64)
    return float(np.dot(u, u)) / u.size


def log_ratio(x, mu_p, mu_q, sigma_p, sigma_q):
    """Eq. 5: the 1/d-scaled Gaussian log likelihood ratio of target over draft at x."""
    x = np.asarray(x, dtype=np.float64)
    return (-energy(x - mu_p) / (2.0 * sigma_p ** 2)
            + energy(x - mu_q) / (2.0 * sigma_q ** 2)
            + 0.5 * math.log(sigma_q ** 2 / sigma_p ** 2))


def log_ratio_diag(x, mu_p, mu_q, s_p, s_q):
    """Remark "General covariances", diagonal case: Eq. 5 with the scaled Euclidean energies
    replaced by scaled Mahalanobis energies (1/d) (x - mu)^T Sigma^-1 (x - mu) and the normalisation
    term by (1/2d) log(|Sigma_q| / |Sigma_p|), Sigma = diag(s^2).  s_p, s_q: per-dimension scales."""
    x, mu_p, mu_q = (np.asarray(a, dtype=np.float64) for a in (x, mu_p, mu_q))
    s_p = np.broadcast_to(np.asarray(s_p, dtype=np.float64), x.shape)
    s_q = np.broadcast_to(np.asarray(s_q, dtype=np.float64), x.shape)
    d = x.size
    maha_p = float(np.sum(((x - mu_p) / s_p) ** 2)) / d
    maha_q = float(np.sum(((x - mu_q) / s_q) ** 2)) / d
    logdet = float(np.sum(np.log(s_q ** 2)) - np.sum(np.log(s_p ** 2)))
    return -0.5 * maha_p + 0.5 * maha_q + logdet / (2.0 * d)


def within_threshold(x, mu_p, sigma_p):
    """Deterministic acceptance of the standalone TiRex-style variant (Table "TiRex configuration",
    row "Acceptance draw"): a proposal passes iff its scaled squared distance from the target's
    prediction, ||x - mu_p||_d^2 = ||x - mu_p||^2 / d, is at most sigma^2 (per-dimension scales:
    the scaled Mahalanobis distance is at most 1)."""
    if np.ndim(sigma_p):
        return energy((x - mu_p) / np.asarray(sigma_p, dtype=np.float64)) <= 1.0
    return energy(x - mu_p) <= sigma_p * sigma_p


def spec_round(Wt, mt, Wd, md, hist, K, sigma_p, sigma_q, u_fn, single_pass=True, alpha_override=None,
               eps_fn=None, sample_proposals=False, fallback_r=0.0, rule="ratio", target_forced=None):
    """One speculative round for one series.

    hist: [n, P] normalised history (context patches then committed patches).
    u_fn(i) -> the uniform for proposal position i (1-based).
    alpha_override: if not None, the acceptance probability of every position is this constant
        (used to test the block-length law under an i.i.d. acceptance rate).
    Sampled variants (Sec. "Fallback Correction and Sampled Variants", "Bonus Patch"):
    eps_fn(stream, i) -> P standard normals for position i; with sample_proposals the draft
    proposes x_i = mu_q^(i) + sigma_q eps (and conditions its next step on that draw); with
    fallback_r = r > 0 the corrected / bonus patch is mu_p^(n+1) + r eps.  The defaults are the
    deployed mean-propagating scheme (x_i = mu_q^(i), t = mu_p^(n+1)).
    sigma_p / sigma_q may be length-P vectors: the diagonal-covariance surrogate (Remark "General
    covariances"); scalars are the isotropic surrogate of Eq. 4.
    rule: "ratio" is the likelihood-ratio test of Eq. 5 against a uniform draw; "threshold" is the
    deterministic test of `within_threshold` (no draw is used).  For the threshold rule the record
    carries the same decision in log form, ell = -||x - mu_p||_d^2 / (2 sigma_p^2) against the
    constant log u = -1/2, so that callers can see how close to the boundary a decision was.
    target_forced: imposed expert choices of a routed target for the positions of hist and the
    proposals ([layers, >= n + K, top_k], see `ffn_routed`; comparison aid, default off).
    Returns a dict with X, mu_q [K, P], mu_p [K+1, P], ell, logu [K] (nan where untested),
    n (accepted count) and commits [n + 1, P].
    """
    if rule not in ("ratio", "threshold"):
        raise ValueError("rule must be 'ratio' or 'threshold'")
    hist = np.asarray(hist, dtype=np.float64)
    P = hist.shape[1]
    X = np.empty((K, P))
    mu_q = np.empty((K, P))
    cur = hist
    sigma_q = np.asarray(sigma_q, dtype=np.float64) if np.ndim(sigma_q) else sigma_q
    for i in range(K):                               # K sequential draft passes
        mu_q[i] = forward(Wd, md, cur)[-1]
        X[i] = mu_q[i] + sigma_q * eps_fn(STREAM_PROPOSAL, i + 1) if sample_proposals else mu_q[i]
        cur = np.vstack([cur, X[i][None, :]])
    n0 = hist.shape[0]
    if single_pass:                                  # one causal pass, read at the K+1 boundaries
        mu_p = forward(Wt, mt, cur, forced_experts=target_forced)[n0 - 1: n0 + K]
    else:                                            # definitional: K+1 separate passes
        mu_p = np.stack([forward(Wt, mt, cur[: n0 + i], forced_experts=target_forced)[-1] for i in range(K + 1)])
    ell = np.full(K, np.nan)
    logu = np.full(K, np.nan)
    n = 0
    for i in range(K):                               # left to right, stop at the first rejection
        if rule == "threshold":
            if np.ndim(sigma_p):
                ell[i] = -0.5 * energy((X[i] - mu_p[i]) / np.asarray(sigma_p, dtype=np.float64))
            else:
                ell[i] = -energy(X[i] - mu_p[i]) / (2.0 * sigma_p * sigma_p)
            logu[i] = -0.5
            if within_threshold(X[i], mu_p[i], sigma_p):
                n += 1
                continue
            break
        if np.ndim(sigma_p) or np.ndim(sigma_q):
            ell[i] = log_ratio_diag(X[i], mu_p[i], mu_q[i], sigma_p, sigma_q)
        else:
            ell[i] = log_ratio(X[i], mu_p[i], mu_q[i], sigma_p, sigma_q)
        logu[i] = math.log(u_fn(i + 1))
        thresh = math.log(alpha_override) if alpha_override is not None else min(0.0, ell[i])
        if logu[i] <= thresh:
            n += 1
        else:
            break
    t = mu_p[n] + fallback_r * eps_fn(STREAM_FALLBACK, n + 1) if fallback_r > 0.0 else mu_p[n]
    commits = np.vstack([X[:n], t[None, :]])         # fallback (n < K) or bonus (n == K)
    return dict(X=X, mu_q=mu_q, mu_p=mu_p, ell=ell, logu=logu, n=n, commits=commits)


def forecast_spec(Wt, mt, Wd, md, series_context, P, horizon, K, sigma_p, sigma_q, seed, b,
                  single_pass=True, alpha_override=None, u_fn=None, trace=None, sample_proposals=False,
                  fallback_r=0.0, round0=0, rule="ratio"):
    """Speculative forecast of one series.  series_context: raw context steps (length N * P).
    Returns (forecast [horizon] in raw units, stats dict).  `trace`, if a list, receives each
    round's record."""
    ctx = np.asarray(series_context, dtype=np.float64)
    m, s = context_stats(ctx)
    hist = ((ctx - m) / s).reshape(-1, P)
    T = -(-horizon // P)
    Y = np.empty((0, P))
    stats = dict(rounds=0, tested=0, accepted=0, committed=0, lengths=[])
    r = round0                                       # the draws' round counter (a reused batch slot keeps counting)
    while Y.shape[0] < T:
        draw = (lambda i, r=r: u_fn(b, r, i)) if u_fn is not None else (lambda i, r=r: uniform(seed, b, r, i))
        eps = lambda stream, i, r=r: normal(seed, b, r, i, stream, P)
        K_r = min(K, T - Y.shape[0])                 # no proposals for patches past the horizon
        rec = spec_round(Wt, mt, Wd, md, np.vstack([hist, Y]), K_r, sigma_p, sigma_q, draw,
                         single_pass=single_pass, alpha_override=alpha_override, eps_fn=eps,
                         sample_proposals=sample_proposals, fallback_r=fallback_r, rule=rule)
        if trace is not None:
            trace.append(rec)
        n = rec["n"]
        stats["rounds"] += 1
        stats["tested"] += n + (1 if n < K_r else 0)
        stats["accepted"] += n
        stats["lengths"].append(n + 1)
        Y = np.vstack([Y, rec["commits"]])[:T]       # whole patches, never more than T (drops a bonus patch at T + 1)
        r += 1
    stats["committed"] = Y.shape[0]
    return (Y.reshape(-1) * s + m)[:horizon], stats


def commit_block(rec, n, fallback_r=0.0, eps_fn=None):
    """The patches a round commits when it keeps n of its proposals: x_1..x_n, then the target's
    prediction at position n + 1 (plus r eps when fallback noise is on)."""
    t = rec["mu_p"][n] + fallback_r * eps_fn(STREAM_FALLBACK, n + 1) if fallback_r > 0.0 else rec["mu_p"][n]
    return np.vstack([rec["X"][:n], t[None, :]])


def forecast_spec_sync(Wt, mt, Wd, md, contexts, P, horizon, K, sigma_p, sigma_q, seed, rule="ratio",
                       single_pass=True, sample_proposals=False, fallback_r=0.0, trace=None):
    """Batch-synchronised speculative forecast (Table "TiRex configuration", acceptance row: the
    batch is kept in step): every round each series runs its own tests, and the whole batch then
    keeps the smallest accepted count among them, so that all series stay at the same length: each
    commits its first n_min proposals and its target's prediction at position n_min + 1.
    contexts: [B, N * P] raw context steps.  Returns (forecasts [B, horizon], list of per-series
    stats).  tested / accepted count each series' own tests (what it tried before its own first
    rejection); committed follows the synchronised length.  `trace`, if a list, receives per round
    the list of the series' records, each with the extra key n_sync."""
    contexts = np.asarray(contexts, dtype=np.float64)
    B = contexts.shape[0]
    T = -(-horizon // P)
    norm = [context_stats(contexts[b]) for b in range(B)]
    hist = [((contexts[b] - norm[b][0]) / norm[b][1]).reshape(-1, P) for b in range(B)]
    Y = [np.empty((0, P)) for _ in range(B)]
    stats = [dict(rounds=0, tested=0, accepted=0, committed=0, lengths=[]) for _ in range(B)]
    r = 0
    while Y[0].shape[0] < T:                         # all series have the same length
        K_r = min(K, T - Y[0].shape[0])
        recs = []
        for b in range(B):
            draw = lambda i, b=b: uniform(seed, b, r, i)
            eps = lambda stream, i, b=b: normal(seed, b, r, i, stream, P)
            recs.append(spec_round(Wt, mt, Wd, md, np.vstack([hist[b], Y[b]]), K_r, sigma_p, sigma_q, draw,
                                   single_pass=single_pass, eps_fn=eps, sample_proposals=sample_proposals,
                                   fallback_r=fallback_r, rule=rule))
        n_sync = min(rec["n"] for rec in recs)
        for b in range(B):
            rec = recs[b]
            rec["n_sync"] = n_sync
            eps = lambda stream, i, b=b: normal(seed, b, r, i, stream, P)
            stats[b]["rounds"] += 1
            stats[b]["tested"] += rec["n"] + (1 if rec["n"] < K_r else 0)
            stats[b]["accepted"] += rec["n"]
            stats[b]["lengths"].append(n_sync + 1)
            Y[b] = np.vstack([Y[b], commit_block(rec, n_sync, fallback_r, eps)])[:T]
        if trace is not None:
            trace.append(recs)
        r += 1
    out = np.empty((B, horizon))
    for b in range(B):
        stats[b]["committed"] = Y[b].shape[0]
        out[b] = (Y[b].reshape(-1) * norm[b][1] + norm[b][0])[:horizon]
    return out, stats


def forecast_target_only(Wt, mt, series_context, P, horizon):
    """Eq. 1: T = ceil(H / P) sequential target passes, each committing the target's mean patch."""
    ctx = np.asarray(series_context, dtype=np.float64)
    m, s = context_stats(ctx)
    hist = ((ctx - m) / s).reshape(-1, P)
    T = -(-horizon // P)
    for _ in range(T):
        hist = np.vstack([hist, forward(Wt, mt, hist)[-1][None, :]])
    return (hist[-T:].reshape(-1) * s + m)[:horizon]


# ----------------------------------------------------------------------------------------------
# Throughput law (Eq. 7, Eq. 8, marginal-gain criterion for K)
# ----------------------------------------------------------------------------------------------
def block_length_pmf(alpha, K):
    """P(L = l), l = 1..K+1, under an i.i.d. per-position acceptance rate alpha."""
    return np.array([(1 - alpha) * alpha ** (l - 1) for l in range(1, K + 1)] + [alpha ** K])


def expected_block_length(alpha, K):
    return float(K + 1) if alpha == 1.0 else (1 - alpha ** (K + 1)) / (1 - alpha)


def predicted_speedup(alpha, K, c, v):
    return expected_block_length(alpha, K) / (c * K + v)


def next_position_pays(alpha, K, c, v):
    """S(K+1) >= S(K)  iff  alpha^(K+1) (cK + v) >= c E[L_K]."""
    return alpha ** (K + 1) * (c * K + v) >= c * expected_block_length(alpha, K)


def choose_block_size(alpha, c, v, k_max):
    """Proposition "Marginal-gain condition for K": S(K+1) >= S(K) iff alpha^(K+1) (cK + v) >= c E[L_K].
    The left side minus the right side falls strictly with K, so S is unimodal; returned is the
    first K at which one more position no longer pays, i.e. the maximiser of S on 1..k_max.  (The
    paper words K* as the largest K for which the condition still holds, which is one less.)"""
    K = 1
    while K < k_max and next_position_pays(alpha, K, c, v):
        K += 1
    return K


def hoeffding_halfwidth(n, delta):
    """Theorem "Hoeffding concentration": with n i.i.d. per-history terms in [0, 1],
    P(|estimate - mean| >= eps) <= 2 exp(-2 n eps^2); the eps at which that bound equals delta."""
    return math.sqrt(math.log(2.0 / delta) / (2.0 * n))
