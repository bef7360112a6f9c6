"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each one compares the oracle with
something that is not the oracle: a closed form of Eq.3-5, an invariant of
Eq.1 / Eq.6, hand-computed numbers (tests/golden/hand_example.txt), numpy's
matmul applied to the textbook top-k MoE, or a brute-force Python loop.
"""
import math
from types import SimpleNamespace as NS

import numpy as np
import pytest

import oracle
from workloads import (WORKLOADS, LayerShape, make_inputs, ffn_work_fraction,
                       n_const_rule)


def shape(T, D, F, n_ffn, n_zero, n_copy, n_const, k=2):
    return NS(T=T, D=D, F=F, n_ffn=n_ffn, n_zero=n_zero, n_copy=n_copy,
              n_const=n_const, k=k, N=n_ffn + n_zero + n_copy + n_const)


def rand_layer(sh, seed, residual=True, wstd=0.3):
    """Random float32 tensors for a small layer (larger weights than the
    benchmark's 0.02 so that every term matters numerically)."""
    r = np.random.default_rng(seed)
    f = lambda *s, std=1.0: (r.standard_normal(s) * std).astype(np.float32)
    inp = dict(x=f(sh.T, sh.D), W_g=f(sh.N, sh.D, std=wstd),
               w1=f(sh.n_ffn, sh.F, sh.D, std=wstd), w3=f(sh.n_ffn, sh.F, sh.D, std=wstd),
               w2=f(sh.n_ffn, sh.D, sh.F, std=wstd), const_vecs=f(sh.n_const, sh.D),
               W_c=f(sh.n_const, 2, sh.D, std=wstd), bias=None)
    if residual:
        inp["prev_gate"] = f(sh.T, sh.N)
        inp["W_res"] = f(sh.N, sh.N, std=wstd)
    else:
        inp["prev_gate"] = inp["W_res"] = None
    return inp


def np_ffn(x, w1, w3, w2):
    """Textbook SwiGLU FFN with numpy matmuls in fp64: x [n,D] -> [n,D]."""
    x = x.astype(np.float64)
    g = x @ w1.astype(np.float64).T
    u = x @ w3.astype(np.float64).T
    return ((g / (1.0 + np.exp(-g))) * u) @ w2.astype(np.float64).T


# ---------------------------------------------------------------- hand examples
def _hand_layer(router_rows, W_c):
    sh = shape(T=1, D=2, F=2, n_ffn=1, n_zero=0, n_copy=1, n_const=1)
    eye = np.eye(2, dtype=np.float32)[None]
    inp = dict(x=np.array([[1.0, 2.0]], np.float32),
               W_g=np.array(router_rows, np.float32), prev_gate=None, W_res=None,
               w1=eye, w3=eye, w2=eye, bias=None,
               const_vecs=np.array([[10.0, 20.0]], np.float32),
               W_c=np.array([W_c], np.float32))
    return sh, inp


def test_hand_example_A_constant_plus_copy(golden):
    g = golden("hand_example.txt")
    sh, inp = _hand_layer([[1, 0], [0, 1], [1, 1]], [[0, 0], [0, 0]])
    r = oracle.layer_forward(sh, inp)
    assert r["out_gate"][0].tolist() == g["A.logits"][0]
    np.testing.assert_allclose(r["probs"][0], g["A.probs"][0], rtol=1e-14)
    assert r["topk_idx"][0].tolist() == [int(v) for v in g["A.topk_idx"][0]]
    np.testing.assert_allclose(r["topk_w"][0], g["A.topk_w"][0], rtol=1e-7)
    # gate weights are float32-rounded, so y carries a 6e-8 relative error
    np.testing.assert_allclose(r["out"][0], g["A.y"][0], rtol=2e-7)
    # the golden numbers really are the closed forms they claim to be
    Z = math.e + math.e ** 2 + math.e ** 3
    np.testing.assert_allclose(g["A.probs"][0], [math.e / Z, math.e ** 2 / Z, math.e ** 3 / Z],
                               rtol=1e-15)
    np.testing.assert_allclose(g["A.y"][0], [math.e ** 3 / Z * 5.5 + math.e ** 2 / Z * 1,
                                             math.e ** 3 / Z * 11 + math.e ** 2 / Z * 2], rtol=1e-15)


def test_hand_example_B_ffn_plus_copy(golden):
    g = golden("hand_example.txt")
    sh, inp = _hand_layer([[1, 1], [0, 1], [1, 0]], [[0, 0], [0, 0]])
    r = oracle.layer_forward(sh, inp, want_slots=True, want_h=True)
    assert r["out_gate"][0].tolist() == g["B.logits"][0]
    assert r["topk_idx"][0].tolist() == [0, 1]
    np.testing.assert_allclose(r["slot_out"][0, 0], g["B.ffn"][0], rtol=1e-14)
    np.testing.assert_allclose(r["slot_out"][0, 1], [1.0, 2.0], rtol=0)
    np.testing.assert_allclose(r["out"][0], g["B.y"][0], rtol=2e-7)
    sig = lambda z: 1 / (1 + math.exp(-z))
    np.testing.assert_allclose(g["B.ffn"][0], [sig(1), 4 * sig(2)], rtol=1e-15)


def test_hand_example_C_constant_alpha(golden):
    g = golden("hand_example.txt")
    sh, inp = _hand_layer([[1, 0], [0, 1], [1, 1]], [[1, 0], [0, 1]])
    r = oracle.layer_forward(sh, inp, want_slots=True, want_alpha=True)
    assert r["topk_idx"][0].tolist() == [2, 1]
    np.testing.assert_allclose(r["alpha1"][0, 0], g["C.alpha1"][0][0], rtol=1e-14)
    np.testing.assert_allclose(r["slot_out"][0, 0], g["C.e_const"][0], rtol=1e-14)


def test_ffn_not_symmetric_in_w1_w3():
    """silu goes on W1 x, not on W3 x; W2 is applied as [D,F] (no transpose)."""
    sh = shape(T=1, D=2, F=3, n_ffn=1, n_zero=1, n_copy=0, n_const=0, k=1)
    w1 = np.array([[[1, 0], [0, 1], [1, 1]]], np.float32)      # [1,F,D]
    w3 = np.array([[[2, 0], [0, 0.5], [1, -1]]], np.float32)
    w2 = np.array([[[1, 2, 3], [0, -1, 4]]], np.float32)       # [1,D,F]
    x = np.array([[1.0, 2.0]], np.float32)
    sig = lambda z: 1 / (1 + math.exp(-z))
    gpre, up = [1.0, 2.0, 3.0], [2.0, 1.0, -1.0]
    h = [gpre[i] * sig(gpre[i]) * up[i] for i in range(3)]
    want = [h[0] + 2 * h[1] + 3 * h[2], -h[1] + 4 * h[2]]
    r = oracle.experts(sh, x, np.array([[0]], np.int32), np.array([[1.0]], np.float32),
                       w1, w3, w2, np.zeros((0, 2), np.float32), np.zeros((0, 2, 2), np.float32),
                       want_h=True)
    np.testing.assert_allclose(r["h"][0, 0], h, rtol=1e-14)
    np.testing.assert_allclose(r["out"][0], want, rtol=1e-14)


# ------------------------------------------------------- zero / copy / constant
def test_copy_only_layer_returns_x():
    """Two copy experts, K = N = 2: the gate weights sum to 1, so y = x (Eq.4)."""
    sh = shape(T=37, D=24, F=8, n_ffn=0, n_zero=0, n_copy=2, n_const=0)
    inp = rand_layer(sh, 1)
    r = oracle.layer_forward(sh, inp)
    np.testing.assert_allclose(r["out"], inp["x"].astype(np.float64), rtol=3e-7, atol=0)


def test_copy_experts_return_weighted_x():
    """Copy-only routing with N > K: y = (sum of selected gate weights) x."""
    sh = shape(T=50, D=16, F=8, n_ffn=0, n_zero=0, n_copy=5, n_const=0)
    inp = rand_layer(sh, 2)
    r = oracle.layer_forward(sh, inp)
    gsum = r["topk_w"].astype(np.float64).sum(1, keepdims=True)
    assert np.all(gsum < 1.0)                      # not renormalised over top-K
    np.testing.assert_allclose(r["out"], gsum * inp["x"], rtol=1e-14)


def test_zero_only_layer_returns_zero():
    sh = shape(T=20, D=16, F=8, n_ffn=0, n_zero=3, n_copy=0, n_const=0)
    r = oracle.layer_forward(sh, rand_layer(sh, 3))
    assert np.all(r["out"] == 0.0)


def test_zero_expert_degrades_top2_to_top1():
    """One FFN + one zero expert, K = 2: y = g_ffn FFN(x) (Sec. 3.1)."""
    sh = shape(T=33, D=12, F=20, n_ffn=1, n_zero=1, n_copy=0, n_const=0)
    inp = rand_layer(sh, 4)
    r = oracle.layer_forward(sh, inp)
    ffn = np_ffn(inp["x"], inp["w1"][0], inp["w3"][0], inp["w2"][0])
    g_ffn = np.where(r["topk_idx"][:, 0] == 0, r["topk_w"][:, 0], r["topk_w"][:, 1])
    np.testing.assert_allclose(r["out"], g_ffn[:, None].astype(np.float64) * ffn,
                               rtol=1e-11, atol=1e-13)


def _const_only(sh, inp):
    idx = np.full((sh.T, 1), sh.n_ffn + sh.n_zero + sh.n_copy, np.int32)
    return oracle.experts(sh, inp["x"], idx, np.ones((sh.T, 1), np.float32), inp["w1"],
                          inp["w3"], inp["w2"], inp["const_vecs"], inp["W_c"],
                          want_alpha=True)


def test_constant_expert_closed_forms():
    sh = shape(T=40, D=10, F=4, n_ffn=1, n_zero=1, n_copy=1, n_const=1, k=1)
    inp = rand_layer(sh, 5)
    x, v = inp["x"].astype(np.float64), inp["const_vecs"][0].astype(np.float64)

    # generic: a1 = sigmoid((W_c[0] - W_c[1]) x), a1 + a2 = 1
    r = _const_only(sh, inp)
    dl = x @ (inp["W_c"][0, 0].astype(np.float64) - inp["W_c"][0, 1].astype(np.float64))
    a1 = 1 / (1 + np.exp(-dl))
    np.testing.assert_allclose(r["alpha1"][:, 0], a1, rtol=1e-12)
    np.testing.assert_allclose(r["out"], a1[:, None] * x + (1 - a1)[:, None] * v, rtol=1e-12,
                               atol=1e-14)

    # W_c = 0 -> (x + v) / 2
    z = dict(inp, W_c=np.zeros_like(inp["W_c"]))
    np.testing.assert_allclose(_const_only(sh, z)["out"], 0.5 * x + 0.5 * v, rtol=1e-15)

    # v = 0 -> a1 x
    z = dict(inp, const_vecs=np.zeros_like(inp["const_vecs"]))
    np.testing.assert_allclose(_const_only(sh, z)["out"], a1[:, None] * x, rtol=1e-12, atol=1e-300)

    # a1 -> 1: the constant expert degenerates to the copy expert; a2 -> 1: to v
    big = np.zeros_like(inp["W_c"])
    xs = np.abs(inp["x"]) + 1.0                    # strictly positive tokens
    big[0, 0, :] = 100.0
    np.testing.assert_allclose(_const_only(sh, dict(inp, x=xs, W_c=big))["out"], xs, rtol=1e-15)
    big[:] = 0
    big[0, 1, :] = 100.0
    np.testing.assert_allclose(_const_only(sh, dict(inp, x=xs, W_c=big))["out"],
                               np.broadcast_to(v, xs.shape), rtol=1e-15)


def test_two_constant_experts_use_their_own_parameters():
    sh = shape(T=30, D=8, F=4, n_ffn=0, n_zero=0, n_copy=0, n_const=2, k=2)
    inp = rand_layer(sh, 6)
    r = oracle.layer_forward(sh, inp, want_slots=True, want_alpha=True)
    x = inp["x"].astype(np.float64)
    for t in range(sh.T):
        for s in range(2):
            j = r["topk_idx"][t, s]
            Wc = inp["W_c"][j].astype(np.float64)
            l = Wc @ x[t]
            a = np.exp(l - l.max()); a /= a.sum()
            want = a[0] * x[t] + a[1] * inp["const_vecs"][j].astype(np.float64)
            np.testing.assert_allclose(r["slot_out"][t, s], want, rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(r["alpha1"][t, j], a[0], rtol=1e-12)


def test_ffn_plus_constant_combination():
    """FFN + constant expert = FFN output adjusted by x and v (Sec. 3.1)."""
    sh = shape(T=25, D=12, F=16, n_ffn=1, n_zero=0, n_copy=0, n_const=1)
    inp = rand_layer(sh, 7)
    r = oracle.layer_forward(sh, inp, want_alpha=True)
    x = inp["x"].astype(np.float64)
    ffn = np_ffn(inp["x"], inp["w1"][0], inp["w3"][0], inp["w2"][0])
    p = r["probs"].astype(np.float32).astype(np.float64)
    a1 = r["alpha1"][:, :1]
    want = p[:, :1] * ffn + p[:, 1:] * (a1 * x + (1 - a1) * inp["const_vecs"][0].astype(np.float64))
    np.testing.assert_allclose(r["out"], want, rtol=1e-10, atol=1e-12)


def test_zero_plus_copy_bypasses_layer():
    sh = shape(T=25, D=12, F=4, n_ffn=0, n_zero=1, n_copy=1, n_const=0)
    inp = rand_layer(sh, 8)
    r = oracle.layer_forward(sh, inp)
    g_copy = r["probs"][:, 1].astype(np.float32).astype(np.float64)
    np.testing.assert_allclose(r["out"], g_copy[:, None] * inp["x"], rtol=1e-14)


def test_w3_zero_gives_zero_and_large_w1_gives_bilinear():
    sh = shape(T=10, D=6, F=8, n_ffn=2, n_zero=0, n_copy=0, n_const=0)
    inp = rand_layer(sh, 9)
    r = oracle.layer_forward(sh, dict(inp, w3=np.zeros_like(inp["w3"])))
    assert np.all(r["out"] == 0.0)
    # silu(z) -> z for large positive z: with x > 0 and W1 large positive the
    # expert is the bilinear form W2((W1 x) * (W3 x))
    xs = np.abs(inp["x"]) + 1.0
    w1 = np.abs(inp["w1"]) * 100 + 50
    r = oracle.experts(sh, xs, np.tile(np.array([[0, 1]], np.int32), (sh.T, 1)),
                       np.ones((sh.T, 2), np.float32), w1, inp["w3"], inp["w2"],
                       inp["const_vecs"], inp["W_c"], want_slots=True)
    x64 = xs.astype(np.float64)
    for e in range(2):
        bil = ((x64 @ w1[e].astype(np.float64).T) * (x64 @ inp["w3"][e].astype(np.float64).T)) \
            @ inp["w2"][e].astype(np.float64).T
        np.testing.assert_allclose(r["slot_out"][:, e], bil, rtol=1e-12)


# --------------------------------------------------------------------- router
def test_router_matches_numpy_and_softmax_sums_to_one():
    sh = shape(T=64, D=48, F=4, n_ffn=5, n_zero=1, n_copy=1, n_const=2)
    inp = rand_layer(sh, 10)
    bias = np.linspace(-1, 1, sh.N).astype(np.float32)
    r = oracle.route(sh, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"], bias,
                     want_probs=True)
    L = (inp["x"].astype(np.float64) @ inp["W_g"].astype(np.float64).T
         + inp["prev_gate"].astype(np.float64) @ inp["W_res"].astype(np.float64).T
         + bias.astype(np.float64))
    np.testing.assert_allclose(r["out_gate"], L, rtol=3e-7, atol=1e-7)
    np.testing.assert_allclose(r["probs"].sum(1), 1.0, rtol=1e-14)
    L32 = r["out_gate"].astype(np.float64)
    sm = np.exp(L32 - L32.max(1, keepdims=True)); sm /= sm.sum(1, keepdims=True)
    np.testing.assert_allclose(r["probs"], sm, rtol=1e-13)
    # Top-K = the K largest logits, descending
    order = np.argsort(-r["out_gate"], axis=1, kind="stable")[:, :sh.k]
    assert np.array_equal(r["topk_idx"], order)
    np.testing.assert_array_equal(r["topk_w"], np.take_along_axis(r["probs"], order, 1).astype(np.float32))


def test_router_W_res_is_applied_untransposed():
    """G = W x + W_g G_prev with W_g on the left (Eq.6): a single non-zero
    entry W_res[i,m] moves G_prev[m] into logit i, not the other way round."""
    sh = shape(T=3, D=4, F=4, n_ffn=3, n_zero=0, n_copy=0, n_const=0, k=1)
    x = np.zeros((3, 4), np.float32)
    W = np.zeros((3, 4), np.float32)
    prev = np.array([[1, 2, 3], [4, 5, 6], [7, 8, 9]], np.float32)
    Wr = np.zeros((3, 3), np.float32)
    Wr[0, 2] = 2.0
    r = oracle.route(sh, x, prev, W, Wr)
    assert r["out_gate"].tolist() == [[6, 0, 0], [12, 0, 0], [18, 0, 0]]


def test_first_layer_equals_zero_residual_matrix():
    sh = shape(T=40, D=16, F=4, n_ffn=4, n_zero=1, n_copy=1, n_const=1)
    inp = rand_layer(sh, 11)
    a = oracle.route(sh, inp["x"], None, inp["W_g"], None)
    b = oracle.route(sh, inp["x"], inp["prev_gate"], inp["W_g"], np.zeros_like(inp["W_res"]))
    for k in a:
        assert np.array_equal(a[k], b[k])
    with pytest.raises(ValueError):
        oracle.route(sh, inp["x"], inp["prev_gate"], inp["W_g"], None)


def test_identity_residual_reproduces_previous_pathway():
    """W = 0 and W_g = I: G(x^j) = G(x^{j-1}), so the token keeps its pathway."""
    sh = shape(T=40, D=16, F=4, n_ffn=4, n_zero=1, n_copy=1, n_const=1)
    inp = rand_layer(sh, 12)
    r = oracle.route(sh, inp["x"], inp["prev_gate"], np.zeros_like(inp["W_g"]),
                     np.eye(sh.N, dtype=np.float32))
    assert np.array_equal(r["out_gate"], inp["prev_gate"])
    assert np.array_equal(r["topk_idx"], np.argsort(-inp["prev_gate"], 1, kind="stable")[:, :2])


def test_router_is_linear_and_shift_invariant():
    sh = shape(T=30, D=16, F=4, n_ffn=4, n_zero=1, n_copy=1, n_const=1)
    inp = rand_layer(sh, 13)
    f = lambda x, p: oracle.route(sh, x, p, inp["W_g"], inp["W_res"])["out_gate"].astype(np.float64)
    x2, p2 = rand_layer(sh, 14)["x"], rand_layer(sh, 14)["prev_gate"]
    np.testing.assert_allclose(f(inp["x"] + x2, inp["prev_gate"] + p2),
                               f(inp["x"], inp["prev_gate"]) + f(x2, p2), atol=2e-5)
    # a constant added to every logit changes neither the selection nor g
    a = oracle.route(sh, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"], want_probs=True)
    b = oracle.route(sh, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"],
                     np.full(sh.N, 3.0, np.float32), want_probs=True)
    assert np.array_equal(a["topk_idx"], b["topk_idx"])
    np.testing.assert_allclose(a["probs"], b["probs"], rtol=1e-5)


def test_ties_go_to_the_lower_index_and_slots_descend():
    sh = shape(T=2, D=2, F=2, n_ffn=2, n_zero=1, n_copy=1, n_const=1, k=3)
    x = np.array([[1, 0], [0, 1]], np.float32)
    W = np.array([[1, 5], [2, 5], [2, 1], [1, 5], [2, 0]], np.float32)
    r = oracle.route(sh, x, None, W, None)
    assert r["topk_idx"].tolist() == [[1, 2, 4], [0, 1, 3]]
    assert np.all(np.diff(r["topk_w"], axis=1) <= 0)


def test_forced_selection_keeps_softmax_weights():
    sh = shape(T=20, D=8, F=4, n_ffn=3, n_zero=1, n_copy=1, n_const=1)
    inp = rand_layer(sh, 15)
    free = oracle.route(sh, inp["x"], None, inp["W_g"], None, want_probs=True)
    forced = np.tile(np.array([[5, 0]], np.int32), (sh.T, 1))
    r = oracle.route(sh, inp["x"], None, inp["W_g"], None, forced_idx=forced)
    assert np.array_equal(r["topk_idx"], forced)
    np.testing.assert_array_equal(r["topk_w"], free["probs"][:, [5, 0]].astype(np.float32))


# ---------------------------------------------------------------- permutation
def test_permutation_invariants_and_brute_force():
    sh = shape(T=97, D=8, F=4, n_ffn=5, n_zero=1, n_copy=1, n_const=2)
    inp = rand_layer(sh, 16)
    idx = oracle.route(sh, inp["x"], None, inp["W_g"], None)["topk_idx"]
    p = oracle.permute(sh, idx)
    flat = idx.reshape(-1)
    assert p["counts"].sum() == sh.T * sh.k
    assert np.array_equal(p["counts"], np.bincount(flat, minlength=sh.N))
    assert p["offsets"][0] == 0
    assert np.array_equal(np.diff(p["offsets"]), p["counts"][:sh.n_ffn])
    R = int(p["offsets"][-1])
    # brute force: sort slots by (expert, slot index), FFN experts only
    slots = [q for q in sorted(range(sh.T * sh.k), key=lambda q: (flat[q], q)) if flat[q] < sh.n_ffn]
    assert p["src_of"][:R].tolist() == slots
    assert np.all(p["src_of"][R:] == -1)
    for q in range(sh.T * sh.k):
        if flat[q] < sh.n_ffn:
            assert p["src_of"][p["row_of"][q]] == q
        else:
            assert p["row_of"][q] == -1
    for e in range(sh.n_ffn):
        seg = p["src_of"][p["offsets"][e]:p["offsets"][e + 1]]
        assert np.all(np.diff(seg) > 0) and np.all(flat[seg] == e)


def test_permutation_with_empty_groups_and_all_zc():
    sh = shape(T=6, D=2, F=2, n_ffn=3, n_zero=1, n_copy=1, n_const=0)
    idx = np.array([[2, 3], [2, 4], [3, 4], [2, 0], [4, 3], [0, 2]], np.int32)
    p = oracle.permute(sh, idx)
    assert p["counts"].tolist() == [2, 0, 4, 3, 3]
    assert p["offsets"].tolist() == [0, 2, 2, 6]
    assert p["src_of"][:6].tolist() == [7, 10, 0, 2, 6, 11]
    assert p["row_of"].tolist() == [2, -1, 3, -1, -1, -1, 4, 0, -1, -1, 1, 5]
    p = oracle.permute(sh, np.full((6, 2), 3, np.int32))
    assert p["offsets"].tolist() == [0, 0, 0, 0] and np.all(p["row_of"] == -1)
    with pytest.raises(ValueError):
        oracle.permute(sh, np.full((6, 2), 5, np.int32))


# ------------------------------------------------------- Eq.1 evaluated whole
@pytest.mark.parametrize("seed,residual", [(20, True), (21, False)])
def test_dense_then_mask_equals_per_slot_path(seed, residual):
    sh = shape(T=48, D=24, F=40, n_ffn=4, n_zero=1, n_copy=1, n_const=2)
    inp = rand_layer(sh, seed, residual)
    r = oracle.layer_forward(sh, inp)
    gate = np.zeros((sh.T, sh.N))
    np.put_along_axis(gate, r["topk_idx"].astype(np.int64), r["topk_w"].astype(np.float64), 1)
    d = oracle.dense(sh, inp["x"], gate, inp["w1"], inp["w3"], inp["w2"], inp["const_vecs"],
                     inp["W_c"])
    np.testing.assert_allclose(r["out"], d, rtol=1e-12, atol=1e-13)
    # every expert type is exercised by this input
    assert set(np.unique(r["topk_idx"])) == set(range(sh.N))


def test_vanilla_moe_against_numpy_dense_evaluation():
    """N_ZC = 0 is the textbook top-K MoE (Eq.1-2): evaluate it with numpy
    matmuls over all experts and mask."""
    sh = shape(T=64, D=32, F=48, n_ffn=6, n_zero=0, n_copy=0, n_const=0)
    inp = rand_layer(sh, 22, residual=False)
    r = oracle.layer_forward(sh, inp)
    x64 = inp["x"].astype(np.float64)
    L = (x64 @ inp["W_g"].astype(np.float64).T).astype(np.float32)
    p = np.exp(L.astype(np.float64) - L.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    top = np.argsort(-L, 1, kind="stable")[:, :2]
    want = np.zeros((sh.T, sh.D))
    for e in range(sh.n_ffn):
        sel = (top == e).any(1)
        ge = p[:, e].astype(np.float32).astype(np.float64) * sel
        want += ge[:, None] * np_ffn(inp["x"], inp["w1"][e], inp["w3"][e], inp["w2"][e])
    assert np.array_equal(r["topk_idx"], top)
    np.testing.assert_allclose(r["out"], want, rtol=1e-10, atol=1e-12)


def test_full_layer_against_numpy_with_all_expert_types():
    """Independent numpy evaluation of a layer with every expert type,
    gating residual and bias."""
    sh = shape(T=80, D=32, F=24, n_ffn=3, n_zero=1, n_copy=1, n_const=2)
    inp = rand_layer(sh, 23)
    inp["bias"] = np.array([0.1, -0.2, 0.0, 0.3, 0.2, -0.1, 0.25], np.float32)
    r = oracle.layer_forward(sh, inp)
    x64 = inp["x"].astype(np.float64)
    L = (x64 @ inp["W_g"].astype(np.float64).T
         + inp["prev_gate"].astype(np.float64) @ inp["W_res"].astype(np.float64).T
         + inp["bias"]).astype(np.float32)
    p = np.exp(L.astype(np.float64) - L.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    top = np.argsort(-L, 1, kind="stable")[:, :2]
    outs = [np_ffn(inp["x"], inp["w1"][e], inp["w3"][e], inp["w2"][e]) for e in range(3)]
    outs += [np.zeros_like(x64), x64]
    for j in range(2):
        l = x64 @ inp["W_c"][j].astype(np.float64).T
        a = np.exp(l - l.max(1, keepdims=True)); a /= a.sum(1, keepdims=True)
        outs.append(a[:, :1] * x64 + a[:, 1:] * inp["const_vecs"][j].astype(np.float64))
    want = np.zeros_like(x64)
    for t in range(sh.T):
        for i in top[t]:
            want[t] += np.float64(np.float32(p[t, i])) * outs[i][t]
    assert np.array_equal(r["topk_idx"], top)
    np.testing.assert_allclose(r["out"], want, rtol=1e-10, atol=1e-12)


# ------------------------------------------- paper's closed forms, workloads
def test_tab1_fraction_and_eq10(golden):
    g = golden("tab1_eq10.txt")
    for tau, nf, nz, frac in g["tab1"]:
        assert ffn_work_fraction(tau, int(nf), int(nz)) == pytest.approx(frac, rel=1e-12)
    for nf, nzero, ncopy, nconst in g["eq10"]:
        assert n_const_rule(int(nf), int(nzero), int(ncopy)) == int(nconst)


def test_unbiased_routing_reaches_ffn_with_fraction_of_tab1():
    """tau = 1 in Tab.1: the share of slots that reach an FFN expert is
    N_FFN / N when routing is unbiased; the seeded 'small' workload must land
    within sampling noise of it."""
    s = WORKLOADS["small"]
    assert s.N == 12 and s.bias == "none"
    inp = make_inputs(s.with_(F=8))               # routing does not read FFN weights
    r = oracle.route(s, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"])
    p = oracle.permute(s, r["topk_idx"])
    share = p["offsets"][-1] / (s.T * s.k)
    assert abs(share - ffn_work_fraction(1.0, s.n_ffn, s.n_zc)) < 0.01
    assert p["counts"].sum() == s.T * s.k


def test_skew_workload_has_the_stated_structure():
    s = WORKLOADS["skew"]
    inp = make_inputs(s.with_(F=8))
    r = oracle.route(s, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"], inp["bias"])
    c = oracle.permute(s, r["topk_idx"])["counts"].astype(np.float64)
    assert abs(c[s.n_ffn:].sum() / c.sum() - 0.5) < 0.03
    assert abs(c[0] / c[1:s.n_ffn].mean() - 4.0) < 0.5


def test_mid_workload_has_ragged_groups():
    s = WORKLOADS["mid"]
    inp = make_inputs(s.with_(F=8))
    r = oracle.route(s, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"], inp["bias"])
    c = oracle.permute(s, r["topk_idx"])["counts"][:s.n_ffn]
    assert c.max() > 8 * max(c.min(), 1)
