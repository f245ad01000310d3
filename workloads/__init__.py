"""Seeded synthetic workloads: network layer tables, random weights/inputs, task sets.

This package is pure data generation.  It holds no convolution, no scheduling
rule and no timing logic; both the HIP library's Python binding and the CPU
oracle receive what it produces as plain arrays and integers.
"""
from .nets import Layer, NETS, build_net, layer_shapes, net_macs, net_params  # noqa: F401
from .tensors import make_weights, make_inputs, fold_bn  # noqa: F401
from .tasksets import TaskSpec, TaskSet, make_taskset, make_paper_taskset, virtual_et_table, HP, LP  # noqa: F401
