"""Seeded synthetic workloads for the failure-remapped MoE layer.

This package only *describes and draws inputs*: layer shapes, activations,
router / expert weights, the static expert placement and the set of failed
ranks.  It contains none of the method's arithmetic (no gating, no map
construction, no dispatch) so that both the CPU oracle's tests and the GPU
harness can draw the very same arrays from it without sharing any logic.
"""
from .configs import LayerConfig, CONFIGS, get_config, scaled
from .gen import (make_placement, draw_x, draw_router, draw_expert, draw_shared,
                  draw_logits, failed_mask, work_dtype)

__all__ = ["LayerConfig", "CONFIGS", "get_config", "scaled", "make_placement",
           "draw_x", "draw_router", "draw_expert", "draw_shared", "draw_logits",
           "failed_mask", "work_dtype"]
