"""Seeded random layer shapes inside the documented limits (N <= 64, K <= 8, at most 8
constant experts, D and F multiples of 8), every one compared with the oracle on all
tokens: routing and permutation bit-exact, outputs and intermediates to the layer
tolerance.  The draw mixes sizes that reach every kernel family (matrix-core and generic
router, few-token router, one-workgroup and chunked permutation, tiled, weight-streaming
and generic FFN) with expert mixes the named workloads do not have (no zero-computation
experts, only zero-computation experts, many constant experts, K up to 8)."""
import numpy as np
import pytest

from workloads import LayerShape, make_inputs

from helpers import check_layer, gpu_forward, make_layer

pytestmark = pytest.mark.gpu


def draw(i):
    rng = np.random.default_rng(9000 + i)
    act = "bf16" if rng.random() < 0.75 else "f32"
    D = int(rng.choice([64, 128, 192, 256, 320, 512, 768, 1000, 1024]))
    F = int(rng.choice([64, 72, 128, 256, 384, 512]))
    n_ffn = int(rng.choice([0, 1, 2, 3, 5, 8, 16, 33, 48]))
    n_zero = int(rng.integers(0, 3))
    n_copy = int(rng.integers(0, 3))
    n_const = int(rng.choice([0, 0, 1, 2, 4, 8]))
    if n_ffn + n_zero + n_copy + n_const == 0:
        n_zero = 1
    N = n_ffn + n_zero + n_copy + n_const
    if N > 64:
        n_ffn -= N - 64
        N = 64
    k = int(min(N, rng.choice([1, 2, 2, 2, 3, 4, 8])))
    T = int(rng.choice([1, 7, 33, 64, 65, 130, 256, 257, 500, 1024, 2050, 3000]))
    return LayerShape("rand%d" % i, T=T, D=D, F=F, n_ffn=n_ffn, n_zero=n_zero, n_copy=n_copy,
                      n_const=n_const, k=k, act=act, residual=bool(rng.random() < 0.8),
                      bias="normal" if rng.random() < 0.5 else "none", seed=7000 + i), bool(rng.random() < 0.5)


@pytest.mark.parametrize("i", range(64))
def test_random_shape_against_the_oracle(i):
    s, with_cap = draw(i)
    print("shape", s, "capacities", with_cap, flush=True)
    inp = make_inputs(s)
    for variant in (0, 1):
        L = make_layer(s)
        cap = L.capacity(s.T, 1.1, 0.75) if with_cap else None
        tau = 0.75 if with_cap else 0.0
        res = gpu_forward(s, inp, variant=variant, layer=L, cap=cap, balance_tau=tau)
        errs = check_layer(s, inp, res, cap=None if cap is None else np.array(cap, np.int32), balance_tau=tau)
        print("  variant", variant, errs, flush=True)


def draw_medium(i):
    rng = np.random.default_rng(9500 + i)
    D = int(rng.choice([256, 512, 1024, 1536]))
    F = int(rng.choice([256, 704, 1408]))
    n_ffn = int(rng.choice([3, 8, 24]))
    n_zero, n_copy = int(rng.integers(0, 2)), int(rng.integers(0, 2))
    n_const = int(rng.choice([0, 2, 6]))
    k = int(rng.choice([1, 2, 2, 4]))
    T = int(rng.choice([5000, 12000, 20000, 33000]))
    return LayerShape("med%d" % i, T=T, D=D, F=F, n_ffn=n_ffn, n_zero=n_zero, n_copy=n_copy,
                      n_const=n_const, k=min(k, n_ffn + n_zero + n_copy + n_const), act="bf16",
                      residual=bool(rng.random() < 0.8),
                      bias=str(rng.choice(["none", "normal"])), seed=7500 + i), bool(rng.random() < 0.5)


@pytest.mark.parametrize("i", range(8))
def test_random_medium_shape_against_the_oracle(i):
    """Sizes at which the tiled GEMM runs several rounds of tiles and the permutation
    has hundreds of chunks; routing and permutation on all tokens, outputs and
    intermediates on a seeded sample of 1024 tokens that covers every selected expert."""
    from helpers import sample_tokens
    s, with_cap = draw_medium(i)
    print("shape", s, "capacities", with_cap, flush=True)
    inp = make_inputs(s)
    L = make_layer(s)
    cap = L.capacity(s.T, 1.1, 0.75) if with_cap else None
    tau = 0.75 if with_cap else 0.0
    res = gpu_forward(s, inp, variant=0, layer=L, cap=cap, balance_tau=tau)
    toks = sample_tokens(s, res["topk_idx"], 1024, seed=11 + i)
    errs = check_layer(s, inp, res, tok_list=toks, cap=None if cap is None else np.array(cap, np.int32),
                       balance_tau=tau)
    print("  ", errs, flush=True)
