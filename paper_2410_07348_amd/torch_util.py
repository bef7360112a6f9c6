"""Plumbing between seeded host tensors and the layer: upload a set of numpy
inputs as torch tensors of the layer's types, make a Layer for a shape.  No
layer arithmetic."""
from __future__ import annotations

import numpy as np

from .binding import Layer

ACT_TENSORS = ("x", "w1", "w3", "w2", "const_vecs")     # activation-typed; the rest is float32


def to_device(shape, inp, device="cuda:0"):
    """dict of numpy arrays (None entries allowed) -> dict of device tensors."""
    import torch
    act = torch.bfloat16 if shape.act == "bf16" else torch.float32
    dev = {}
    for name, a in inp.items():
        if a is None:
            dev[name] = None
            continue
        t = torch.from_numpy(np.ascontiguousarray(a))
        if name in ACT_TENSORS:
            t = t.to(act)
        dev[name] = t.to(device)
    return dev


def make_layer(shape, device="cuda:0", T_max=None):
    """A Layer context for a shape object with T, D, F, n_ffn, n_zero, n_copy,
    n_const, k, act."""
    return Layer(T_max or max(shape.T, 1), shape.D, shape.F, shape.n_ffn, shape.n_zero,
                 shape.n_copy, shape.n_const, k=shape.k, act=shape.act, device=device)
