"""Pins of the oracle's expert-capacity and load-balance functions (Sec. 3.3,
Eq.7 and Eq.8) against numbers worked by hand (tests/golden/capacity_example.txt),
exact rational arithmetic, the textbook token-dropping rule they reduce to,
a brute-force Python walk, numpy reductions and closed forms.  No HIP code."""
import math
from fractions import Fraction
from types import SimpleNamespace as NS

import numpy as np
import pytest

import oracle
from test_oracle_pins import rand_layer, shape


def ivec(row):
    return np.array(row, dtype=np.int64)


def test_capacity_hand_example(golden):
    g = golden("capacity_example.txt")
    sh = shape(T=5, D=8, F=8, n_ffn=2, n_zero=1, n_copy=1, n_const=0)
    cap = oracle.capacity(sh, 1.0, 0.5)
    assert np.array_equal(cap, ivec(g["CAP.cap"][0]))
    idx = ivec(g["CAP.topk_idx"][0]).reshape(5, 2)
    r = oracle.permute_capacity(sh, idx, cap)
    for key in ("counts", "kept", "offsets", "row_of"):
        assert np.array_equal(r[key], ivec(g["CAP." + key][0])), key
    R = int(r["offsets"][-1])
    assert np.array_equal(r["src_of"][:R], ivec(g["CAP.src_of"][0]))


def test_eq8_at_the_papers_defaults(golden):
    g = golden("capacity_example.txt")
    sh = shape(T=32768, D=8, F=8, n_ffn=16, n_zero=1, n_copy=1, n_const=2)
    cap = oracle.capacity(sh, 1.1, 0.75)
    assert set(cap[:16]) == {int(g["EQ8.c_ffn"][0][0])}
    assert set(cap[16:]) == {int(g["EQ8.c_zc"][0][0])}
    lit = oracle.capacity(sh, 1.1, 0.75, per_assignment=False)
    assert set(lit[:16]) == {int(g["EQ8.lit_c_ffn"][0][0])}
    assert set(lit[16:]) == {int(g["EQ8.lit_c_zc"][0][0])}


@pytest.mark.parametrize("T,k,n_ffn,n_zc,gamma,tau", [
    (100, 2, 8, 4, Fraction(11, 10), Fraction(3, 4)), (7, 3, 5, 2, Fraction(1), Fraction(1, 10)),
    (4096, 2, 16, 4, Fraction(5, 4), Fraction(1, 2)), (33, 1, 3, 0, Fraction(2), Fraction(1)),
    (1000, 4, 1, 7, Fraction(1), Fraction(1, 4))])
def test_eq8_in_exact_rational_arithmetic(T, k, n_ffn, n_zc, gamma, tau):
    """C_i with fractions (no rounding anywhere) and the budget they add up to."""
    sh = shape(T=T, D=8, F=8, n_ffn=n_ffn, n_zero=n_zc, n_copy=0, n_const=0, k=k)
    cap = oracle.capacity(sh, float(gamma), float(tau))
    S, den = T * k, tau * n_ffn + n_zc
    assert all(int(c) == math.ceil(gamma * tau * S / den) for c in cap[:n_ffn])
    assert all(int(c) == math.ceil(gamma * S / den) for c in cap[n_ffn:])
    # the capacities of all experts together offer gamma * S places, rounded up per expert
    assert gamma * S <= int(cap.sum()) < gamma * S + (n_ffn + n_zc)
    # tau is the ratio between the two kinds (up to the rounding)
    if n_zc and n_ffn:
        assert abs(int(cap[0]) - tau * int(cap[-1])) < 1 + tau
    # Eq.8 as it is printed, with the number of tokens T in place of the assignments
    lit = oracle.capacity(sh, float(gamma), float(tau), per_assignment=False)
    assert all(int(c) == math.ceil(gamma * tau * T / den) for c in lit[:n_ffn])
    assert all(int(c) == math.ceil(gamma * T / den) for c in lit[n_ffn:])
    assert gamma * T <= int(lit.sum()) < gamma * T + (n_ffn + n_zc)


def test_without_zero_computation_experts_it_is_the_textbook_capacity():
    """tau = 1, N_ZC = 0: C = ceil(gamma * S / N), the token-dropping rule of
    the vanilla MoE the paper builds on."""
    for T, k, N, gamma in ((64, 2, 8, 1.25), (100, 1, 7, 1.0), (4096, 2, 16, 1.1)):
        sh = shape(T=T, D=8, F=8, n_ffn=N, n_zero=0, n_copy=0, n_const=0, k=k)
        assert set(oracle.capacity(sh, gamma, 1.0)) == {math.ceil(gamma * T * k / N - 1e-9)}


def test_capacity_rejects_nonpositive_parameters():
    sh = shape(T=8, D=8, F=8, n_ffn=2, n_zero=1, n_copy=0, n_const=0)
    for gamma, tau in ((0.0, 1.0), (1.0, 0.0), (-1.0, 0.5)):
        with pytest.raises(ValueError):
            oracle.capacity(sh, gamma, tau)


def random_selection(sh, seed):
    rng = np.random.default_rng(seed)
    return np.stack([rng.permutation(sh.N)[:sh.k] for _ in range(sh.T)]).astype(np.int32)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_permute_capacity_against_a_brute_force_walk(seed):
    sh = shape(T=97, D=8, F=8, n_ffn=4, n_zero=1, n_copy=1, n_const=1, k=3)
    idx = random_selection(sh, seed)
    cap = np.random.default_rng(seed + 10).integers(0, 60, sh.N).astype(np.int32)
    r = oracle.permute_capacity(sh, idx, cap)
    seen = [0] * sh.N
    rows = [[] for _ in range(sh.n_ffn)]
    expect = []
    for q, e in enumerate(idx.reshape(-1).tolist()):        # (token, slot) order
        if seen[e] >= cap[e]:
            expect.append(-2)
        elif e < sh.n_ffn:
            expect.append(None)
            rows[e].append(q)
        else:
            expect.append(-1)
        seen[e] += 1
    flat = [q for lst in rows for q in lst]                 # groups in expert order
    for row, q in enumerate(flat):
        expect[q] = row
    assert r["row_of"].tolist() == expect
    assert r["src_of"][:len(flat)].tolist() == flat
    assert r["counts"].tolist() == seen
    assert r["kept"].tolist() == [min(c, int(k)) for c, k in zip(seen, cap)]
    assert r["offsets"].tolist() == np.concatenate([[0], np.cumsum(r["kept"][:sh.n_ffn])]).tolist()


def test_capacity_that_is_never_reached_changes_nothing():
    sh = shape(T=64, D=8, F=8, n_ffn=3, n_zero=1, n_copy=1, n_const=1)
    idx = random_selection(sh, 5)
    a = oracle.permute(sh, idx)
    b = oracle.permute_capacity(sh, idx, np.full(sh.N, sh.T * sh.k, np.int32))
    for key in ("counts", "offsets", "row_of"):
        assert np.array_equal(a[key], b[key]), key
    assert np.array_equal(b["kept"], b["counts"])
    R = int(a["offsets"][-1])
    assert np.array_equal(a["src_of"][:R], b["src_of"][:R])


def test_dropped_assignments_contribute_nothing():
    """y with capacities = sum over the kept assignments of g * E(x), the
    E(x) taken from a run without capacities; zero capacity gives y = 0."""
    sh = shape(T=40, D=6, F=5, n_ffn=3, n_zero=1, n_copy=1, n_const=1)
    inp = rand_layer(sh, 21)
    full = oracle.layer_forward(sh, inp, want_slots=True)
    cap = np.array([7, 20, 3, 5, 9, 2], np.int32)
    r = oracle.layer_forward(sh, inp, cap=cap)
    assert np.array_equal(r["topk_idx"], full["topk_idx"])
    keep = (r["row_of"].reshape(sh.T, sh.k) != -2)
    assert keep.sum() < sh.T * sh.k and keep.sum() == r["kept"].sum()
    want = np.einsum("tk,tkd->td", full["topk_w"].astype(np.float64) * keep, full["slot_out"])
    assert np.allclose(r["out"], want, rtol=1e-12, atol=1e-12)
    zero = oracle.layer_forward(sh, inp, cap=np.zeros(sh.N, np.int32))
    assert not zero["out"].any() and zero["offsets"][-1] == 0
    assert (zero["row_of"] == -2).all()


def test_balance_hand_example(golden):
    g = golden("capacity_example.txt")
    sh = shape(T=2, D=8, F=8, n_ffn=2, n_zero=1, n_copy=0, n_const=0)
    r = oracle.balance(sh, np.array(g["BAL.probs"][0]).reshape(2, 3),
                       ivec(g["BAL.topk_idx"][0]).reshape(2, 2), 0.5)
    assert np.allclose(r["f"], g["BAL.f"][0], rtol=0, atol=1e-15)
    assert np.allclose(r["P"], g["BAL.P"][0], rtol=0, atol=1e-15)
    assert abs(r["loss"] - g["BAL.loss"][0][0]) < 1e-15


def test_balance_against_numpy_reductions_and_invariants():
    sh = shape(T=300, D=16, F=8, n_ffn=5, n_zero=1, n_copy=1, n_const=2)
    inp = rand_layer(sh, 33)
    r = oracle.route(sh, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"], want_probs=True)
    tau = 0.75
    b = oracle.balance(sh, r["probs"], r["topk_idx"], tau)
    f = np.bincount(r["topk_idx"].reshape(-1), minlength=sh.N) / sh.T
    P = r["probs"].mean(axis=0)
    assert np.allclose(b["f"], f, rtol=0, atol=1e-15) and np.allclose(b["P"], P, rtol=1e-13)
    eta = np.where(np.arange(sh.N) < sh.n_ffn, 1.0, tau)
    assert abs(b["loss"] - float((eta * f * P).sum())) < 1e-13
    assert abs(b["f"].sum() - sh.k) < 1e-12       # every token selects K distinct experts
    assert abs(b["P"].sum() - 1.0) < 1e-12        # softmax rows sum to one
    # tau = 1 is the load-balance loss of a vanilla MoE (without its factor N)
    assert abs(oracle.balance(sh, r["probs"], r["topk_idx"], 1.0)["loss"] - float((f * P).sum())) < 1e-13


def test_balance_closed_form_for_a_router_that_cannot_tell_experts_apart():
    """W = 0, no residual: all logits equal, Softmax = 1/N, ties go to the K
    lowest indices -> f_i = 1 for i < K, P_i = 1/N, L_b = sum_{i<K} eta_i / N."""
    sh = shape(T=50, D=8, F=4, n_ffn=1, n_zero=1, n_copy=1, n_const=1, k=3)
    inp = rand_layer(sh, 8, residual=False)
    inp["W_g"][:] = 0
    r = oracle.route(sh, inp["x"], None, inp["W_g"], None, want_probs=True)
    b = oracle.balance(sh, r["probs"], r["topk_idx"], 0.25)
    assert np.allclose(b["f"], [1, 1, 1, 0]) and np.allclose(b["P"], 0.25)
    assert abs(b["loss"] - (1.0 + 0.25 + 0.25) / 4) < 1e-15
