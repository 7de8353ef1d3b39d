"""Seeded synthetic series with the structure of the benchmark workloads.

Each recipe returns float32 [B, n_steps].  Constants in brackets in the recipes below are
this build's choices where the workload description leaves them open.
"""
import numpy as np


def _seasonal(rng, B, n, n_sines=3):
    t = np.arange(n)[None, :]
    y = np.zeros((B, n))
    for _ in range(n_sines):
        period = rng.integers(12, 337, size=(B, 1))
        amp = rng.uniform(0.5, 1.5, size=(B, 1))
        phase = rng.uniform(0, 2 * np.pi, size=(B, 1))
        y += amp * np.sin(2 * np.pi * t / period + phase)
    return y


def make_series(kind, B, n_steps, seed, n_context_steps=None):
    rng = np.random.default_rng(seed)
    n = n_steps
    t = np.arange(n)[None, :]
    if kind == "two_sines":
        # periods 24 and 168, linear trend, N(0, 0.1) noise, z-normalised over the context
        a = rng.uniform(0.5, 1.5, size=(B, 2, 1))
        ph = rng.uniform(0, 2 * np.pi, size=(B, 2, 1))
        beta = rng.uniform(-1, 1, size=(B, 1))
        y = a[:, 0] * np.sin(2 * np.pi * t / 24 + ph[:, 0]) + a[:, 1] * np.sin(2 * np.pi * t / 168 + ph[:, 1])
        y = y + beta * t / n + 0.1 * rng.standard_normal((B, n))
        c = n_context_steps or n
        y = (y - y[:, :c].mean(1, keepdims=True)) / y[:, :c].std(1, keepdims=True)
    elif kind in ("seasonal_walk_t", "seasonal_walk_t_shift"):
        # 3 sinusoids with periods U{12..336}, random walk (step std 0.05), 0.2 * Student-t(3) noise
        y = _seasonal(rng, B, n)
        y += np.cumsum(0.05 * rng.standard_normal((B, n)), axis=1)
        y += 0.2 * rng.standard_t(3, size=(B, n))
        if kind.endswith("_shift"):
            # 10% of the series get one level shift of N(0, 2) at a uniformly random position
            shifted = rng.random(B) < 0.10
            pos = rng.integers(0, n, size=B)
            step = 2.0 * rng.standard_normal(B)
            y += (shifted[:, None] & (t >= pos[:, None])) * step[:, None]
    elif kind == "smooth_noisy_mix":
        # Bernoulli(1/2) mixture: smooth seasonal (noise std 0.05) or high-noise (noise std 1.0)
        y = _seasonal(rng, B, n)
        noisy = rng.random(B) < 0.5
        y += np.where(noisy[:, None], 1.0, 0.05) * rng.standard_normal((B, n))
    else:
        raise ValueError(f"unknown series kind {kind!r}")
    return y.astype(np.float32)
