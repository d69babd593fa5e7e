"""Seeded synthetic inputs and plain-data model descriptions.

This package is the only code shared by the CPU oracle and the HIP path.  It
holds no arithmetic of the training method: only configuration records (which
layers, which heads, which optimizer) and seeded random generators for
minibatches and initial weights.
"""
from .configs import (LayerCfg, HeadCfg, OptCfg, ModelCfg, make_config,
                      CONFIG_NAMES, param_shapes, head_windows)
from .data import make_batch, init_params, perturb_params, zipf_pmf, zipf_tokens

__all__ = ["LayerCfg", "HeadCfg", "OptCfg", "ModelCfg", "make_config",
           "CONFIG_NAMES", "param_shapes", "head_windows", "make_batch",
           "init_params", "perturb_params", "zipf_pmf", "zipf_tokens"]
