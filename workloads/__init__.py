"""Seeded synthetic inputs for the MoE++ layer forward.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests / benchmark.  It holds layer *shapes* and random tensors; it
evaluates nothing of the layer itself (no router, no experts, no combine).

Shapes follow the model table of the paper (Tab.2: top-2 routing, FFN experts
plus 1 zero / 1 copy / 2 constant experts, sequences of 2048 tokens) scaled to
the hidden sizes the benchmark configurations name.  All random numbers come
from numpy's counter-based Philox generator, one independent stream per
tensor, so a tensor's bytes depend only on (seed, tensor name, shape).
"""
from .gen import (LayerShape, WORKLOADS, PAPER_MODELS, make_inputs, make_router_bias,
                  skew_bias_gaussian_model, round_to_bf16, TENSOR_IDS,
                  ffn_work_fraction, n_const_rule)

__all__ = ["LayerShape", "WORKLOADS", "PAPER_MODELS", "make_inputs", "make_router_bias",
           "skew_bias_gaussian_model", "round_to_bf16", "TENSOR_IDS",
           "ffn_work_fraction", "n_const_rule"]
