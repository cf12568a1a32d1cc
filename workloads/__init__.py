"""Seeded synthetic input generators (graphs, training sets, features, minibatches)."""
from .synth import *  # noqa: F401,F403
from .synth import CONFIGS, TINY, MID, LARGE, WIDE, SKEW, WorkloadConfig, Graph  # noqa: F401
