"""Seeded synthetic workloads: network shape tables and input generators.

This package holds no arithmetic of the training method.  It only describes
the five benchmark networks as neutral layer lists and draws the random
inputs, labels and initial parameters that both the CPU oracle and the HIP
path are fed with, so that neither has to reproduce the other's random
number generator.
"""
from .configs import CONFIGS, get_config, Config  # noqa: F401
from .synth import init_params, make_batch, to_bf16_grid  # noqa: F401
