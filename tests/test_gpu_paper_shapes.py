"""Parity at the layer shapes of the paper's own models (Tab.2): hidden 768 /
intermediate 2048 with 8, 16 or 32 FFN experts, hidden 1536 / intermediate 4096
with 16; zero / copy / constant experts 1/1/2 (1/1/6 with 32 FFN experts), Top-2,
16 sequences of 2048 tokens.  Each layer runs as `bench.py --tau-sweep` runs it:
a router bias under which the zero-computation experts take N_ZC / (tau N_FFN +
N_ZC) of the assignments (Tab.1), the expert capacities of Eq.8 at gamma = 1.1
and the load-balance statistics of Eq.7 on, the MFMA kernels required.
Routing, counts, kept rows and the permutation are compared with the oracle on
all 32768 tokens; out, h and yffn on all tokens for the 768-wide models and on
a seeded sample of 8192 tokens that covers every selected expert for the
1536-wide one (its oracle pass over all tokens takes most of a minute).
The vanilla comparison layer of the sweep (no zero-computation experts, no
capacities) is checked the same way.  Needs a real MI355X: run with -m gpu."""
import numpy as np
import pytest

import oracle
from workloads import PAPER_MODELS, make_inputs, ffn_work_fraction

from helpers import check_layer, gpu_forward, make_layer, sample_tokens

pytestmark = pytest.mark.gpu

GAMMA = 1.1


def say(*a):
    print(*a, flush=True)


def n_sample(shape):
    return None if shape.D <= 768 else 8192


@pytest.mark.parametrize("tau", [0.1, 0.75, 1.0])
@pytest.mark.parametrize("model", sorted(PAPER_MODELS))
def test_paper_model_layer_with_tau_bias_and_capacity(model, tau):
    s = PAPER_MODELS[model].with_(bias="tau%g" % tau)
    say("paper layer", model, "tau", tau, s)
    inp = make_inputs(s)
    L = make_layer(s)
    cap = L.capacity(s.T, GAMMA, tau)
    assert cap == oracle.capacity(s, GAMMA, tau).tolist()
    res = gpu_forward(s, inp, variant=2, layer=L, cap=cap, balance_tau=tau)
    say("gpu done: R", int(res["offsets"][-1]), "counts", res["counts"].tolist(), "cap", cap[0], cap[-1])
    ns = n_sample(s)
    toks = None if ns is None else sample_tokens(s, res["topk_idx"], ns, seed=s.seed)
    errs = check_layer(s, inp, res, tok_list=toks, cap=np.array(cap, np.int32), balance_tau=tau)
    say(model, tau, "errs", errs)
    # the bias steers the zero-computation experts to the share of Tab.1 (seeded
    # Gaussian calibration, so only approximately)
    zc_share = res["counts"][s.n_ffn:].sum() / (s.T * s.k)
    assert abs(zc_share - (1.0 - ffn_work_fraction(tau, s.n_ffn, s.n_zc))) < 0.05
    assert np.all(res["kept"] <= np.array(cap))


@pytest.mark.parametrize("model", sorted(PAPER_MODELS))
def test_paper_model_vanilla_layer(model):
    base = PAPER_MODELS[model]
    s = base.with_(name=base.name + "_vanilla", n_zero=0, n_copy=0, n_const=0)
    say("vanilla layer", model, s)
    inp = make_inputs(s)
    res = gpu_forward(s, inp, variant=2)
    ns = n_sample(s)
    toks = None if ns is None else sample_tokens(s, res["topk_idx"], ns, seed=s.seed)
    errs = check_layer(s, inp, res, tok_list=toks)
    say(model, "vanilla errs", errs)
    assert errs["R"] == s.T * s.k
