"""Seeded synthetic inputs for the merged multi-task (MT) BERT serving forward pass.

This module serves both the CPU oracle and the HIP library and therefore holds none of the
method's arithmetic: it only describes model shapes and draws numbers.  Everything is produced
by one counter-based generator (splitmix64 -> uniform -> Box-Muller), so any tensor can be
regenerated independently from (seed, tensor index).

Model shapes stand in for the paper's workloads (Section 4: eight GLUE tasks on the 12-layer
uncased BERT; Appendix E: the industrial deployment); neither dataset nor checkpoint is needed
because the forward pass is shape-, not value-, dependent.
"""
from .spec import MTSpec, TaskSpec, CONFIGS, get_config, trunk_tensors, task_tensors, layer_tensors
from .gen import (splitmix64, uniform01, normal, make_trunk_params, make_task_params,
                  make_inputs, round_to_bf16_grid, round_to_e4m3_grid, round_group_to_e4m3_grid, e4m3_scale)

__all__ = ["MTSpec", "TaskSpec", "CONFIGS", "get_config", "trunk_tensors", "task_tensors",
           "layer_tensors", "splitmix64", "uniform01", "normal", "make_trunk_params",
           "make_task_params", "make_inputs", "round_to_bf16_grid", "round_to_e4m3_grid", "round_group_to_e4m3_grid", "e4m3_scale"]
