"""Seeded synthetic workloads (shapes and random inputs only; no model arithmetic)."""
from .configs import CONFIGS, CONFIG_ORDER, StageConfig
from . import generate

__all__ = ["CONFIGS", "CONFIG_ORDER", "StageConfig", "generate"]
