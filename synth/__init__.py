"""Seeded synthetic inputs (configurations, weights, series) shared by the CPU oracle's tests
and the GPU harness.  This package holds no arithmetic of the speculative-decoding method:
only random-number recipes, array shapes and the storage rounding of inputs."""
from .configs import ModelCfg, RunCfg, get_config, CONFIGS  # noqa: F401
from .weights import make_weights, weight_spec, flatten_weights, round_to_bf16  # noqa: F401
from .series import make_series  # noqa: F401
from .cases import Inputs  # noqa: F401
