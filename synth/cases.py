"""One configuration's seeded inputs (weights of both models, raw series) in one object."""
import dataclasses

import numpy as np

from .configs import get_config
from .series import make_series
from .weights import make_weights


class Inputs:
    """cfg, wt / wd (dicts of float32 tensors, already rounded to bf16 for bf16 runs), series
    [B, context + horizon] and its context part."""

    def __init__(self, name, B=None, sigma=None, K=None, horizon=None, random_gains=False, draft_is_target=False,
                 seed=2021, **over):
        cfg = get_config(name, **over)
        cfg = dataclasses.replace(cfg, K=K or cfg.K, horizon=horizon or cfg.horizon, sigma=sigma or cfg.sigma,
                                  batch=B or cfg.batch)
        if draft_is_target:
            cfg = dataclasses.replace(cfg, draft=cfg.target)
        self.cfg = cfg
        self.seed = seed          # Philox key of the acceptance draws
        rng = np.random.default_rng(cfg.weight_seed)
        self.wt = make_weights(cfg.target, cfg.patch, rng, cfg.dtype, random_gains=random_gains)
        self.wd = self.wt if draft_is_target else make_weights(cfg.draft, cfg.patch, rng, cfg.dtype,
                                                               random_gains=random_gains)
        self.series = make_series(cfg.series_kind, cfg.batch, cfg.context + cfg.horizon, cfg.series_seed, cfg.context)
        self.context = np.ascontiguousarray(self.series[:, : cfg.context])
