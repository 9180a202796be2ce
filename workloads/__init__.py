"""Seeded synthetic inputs for the SSM-layer prefill workloads.

This package only draws random numbers and rounds them to the storage dtype;
it holds none of the scan's arithmetic, so both the CPU oracle's tests and the
GPU path's tests may take their inputs from it.
"""
from .gen import (  # noqa: F401
    CONFIGS,
    LayerShape,
    Workload,
    draw_layer_inputs,
    make_workload,
)
