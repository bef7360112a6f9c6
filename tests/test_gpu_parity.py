"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element, on seeded inputs.  Needs a real MI355X: run with -m gpu."""
import numpy as np
import pytest

import oracle
from workloads import WORKLOADS, LayerShape, make_inputs

from helpers import (check_layer, gpu_forward, make_layer, sample_tokens, to_device, rel_err,
                     TOL_OUT)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def small_shape(name, **kw):
    base = dict(T=300, D=256, F=384, n_ffn=5, n_zero=1, n_copy=1, n_const=2, k=2,
                act="bf16", seed=77)
    base.update(kw)
    return LayerShape(name, **base)


def forced_routing(shape, idx, seed=5):
    """Inputs whose routing is dictated: W = 0 and W_g (residual) = I, so
    G(x) = G(x_prev) exactly (Eq.6) and prev_gate decides the Top-K."""
    inp = make_inputs(shape.with_(residual=True, bias="none"))
    N = shape.N
    rng = np.random.default_rng(seed)
    pg = (-10.0 + rng.random((shape.T, N))).astype(np.float32)
    for s in range(shape.k):
        pg[np.arange(shape.T), idx[:, s]] = 10.0 - s
    inp["prev_gate"] = pg
    inp["W_g"] = np.zeros((N, shape.D), np.float32)
    inp["W_res"] = np.eye(N, dtype=np.float32)
    inp["bias"] = None
    return inp


# ----------------------------------------------------------------- small cases
def test_tiny_fp32_workload_all_tokens():
    s = WORKLOADS["tiny"]
    inp = make_inputs(s)
    say("case tiny fp32", s)
    res = gpu_forward(s, inp)
    errs = check_layer(s, inp, res)
    say("tiny errs", errs)
    assert set(np.unique(res["topk_idx"])) == set(range(s.N))


@pytest.mark.parametrize("variant", [1, 0])
@pytest.mark.parametrize("kw", [
    dict(),                                            # several tiles + ragged tail
    dict(T=1000, D=512, F=640, n_ffn=7, seed=78),
    dict(T=257, D=128, F=64, n_ffn=3, n_const=1, seed=79),
    dict(T=129, D=192, F=320, n_ffn=6, n_const=3, k=3, seed=80),   # D, F not multiples of 128
    dict(T=64, D=64, F=64, n_ffn=2, n_zero=0, n_copy=0, n_const=0, k=1, seed=81),
    dict(T=2000, D=256, F=256, n_ffn=20, n_zero=0, n_copy=0, n_const=0, seed=82),  # vanilla
    dict(T=500, D=256, F=128, n_ffn=4, n_zero=2, n_copy=2, n_const=4, k=4, seed=83),
    dict(T=333, D=256, F=384, residual=False, seed=84),             # first layer, Eq.6 j = 1
    dict(T=333, D=256, F=384, bias="normal", seed=85),
    dict(T=96, D=1024, F=2048, n_ffn=8, seed=86),
])
def test_bf16_layers_all_tokens(kw, variant):
    s = small_shape("case", **kw)
    inp = make_inputs(s)
    say("case", kw, "variant", variant)
    res = gpu_forward(s, inp, variant=variant)
    say("errs", check_layer(s, inp, res))


@pytest.mark.parametrize("act", ["bf16", "f32"])
@pytest.mark.parametrize("kw", [
    # the limits of the descriptor: N = 64 experts, K = 8 slots, 8 constant experts
    dict(T=300, D=256, F=128, n_ffn=52, n_zero=2, n_copy=2, n_const=8, k=8, seed=95),
    # the widest router the MFMA kernel takes: N + 2 n_const = 64 rows of weights
    dict(T=300, D=256, F=128, n_ffn=38, n_zero=1, n_copy=1, n_const=8, k=8, seed=96),
    # as many FFN experts as the descriptor allows, no other kind
    dict(T=400, D=128, F=64, n_ffn=60, n_zero=0, n_copy=0, n_const=0, k=6, seed=97),
])
def test_maximum_expert_counts(kw, act):
    s = small_shape("max", act=act, **kw)
    inp = make_inputs(s)
    say("max counts", kw, act)
    for variant in ((1, 0) if act == "bf16" else (0,)):
        res = gpu_forward(s, inp, variant=variant)
        say("errs", check_layer(s, inp, res))


@pytest.mark.parametrize("kw", [
    dict(T=200, D=64, F=96, seed=90),
    dict(T=50, D=8, F=8, n_ffn=2, n_const=1, seed=91),             # smallest legal D, F
    dict(T=130, D=72, F=40, n_ffn=3, k=3, seed=92),                # F % 32 != 0 (partial pack block)
])
def test_fp32_layers_all_tokens(kw):
    s = small_shape("case32", act="f32", **kw)
    inp = make_inputs(s)
    say("case fp32", kw)
    res = gpu_forward(s, inp)
    say("errs", check_layer(s, inp, res))


# ------------------------------------------- expert capacity, load balance
@pytest.mark.parametrize("variant", [1, 0])
@pytest.mark.parametrize("kw,gamma,tau", [
    (dict(T=1000, D=256, F=384, n_ffn=6, seed=101), 1.1, 0.75),      # the paper's defaults
    (dict(T=777, D=256, F=128, n_ffn=4, n_zero=2, n_copy=2, n_const=4, k=4, seed=102), 0.5, 0.25),
    (dict(T=600, D=128, F=128, n_ffn=8, n_zero=0, n_copy=0, n_const=0, seed=103), 0.8, 1.0),
    (dict(T=300, D=256, F=256, bias="normal", seed=104), 1.0, 0.1),
    (dict(T=2500, D=128, F=128, n_ffn=6, seed=105), 0.9, 0.5),     # three-kernel permutation
])
def test_expert_capacity_and_balance_statistics(kw, gamma, tau, variant):
    s = small_shape("cap", **kw)
    inp = make_inputs(s)
    L = make_layer(s)
    cap = L.capacity(s.T, gamma, tau)
    assert cap == oracle.capacity(s, gamma, tau).tolist()
    say("capacity", kw, gamma, tau, cap, "variant", variant)
    res = gpu_forward(s, inp, variant=variant, layer=L, cap=cap, balance_tau=tau)
    errs = check_layer(s, inp, res, cap=np.array(cap, np.int32), balance_tau=tau)
    say("errs", errs)
    assert errs["dropped"] > 0
    assert np.all(res["kept"] <= np.array(cap))
    # switching the capacities off again restores the unlimited layer
    res2 = gpu_forward(s, inp, variant=variant, layer=L)
    check_layer(s, inp, res2)
    assert (res2["row_of"] != -2).all()


def test_capacity_extremes():
    s = small_shape("cap0", T=200, n_ffn=4)
    inp = make_inputs(s)
    L = make_layer(s)
    # nothing fits anywhere: every slot is dropped, the layer outputs zero
    res = gpu_forward(s, inp, layer=L, cap=[0] * s.N)
    assert (res["row_of"] == -2).all() and res["offsets"][-1] == 0 and not res["kept"].any()
    assert not res["out"].any()
    check_layer(s, inp, res, cap=np.zeros(s.N, np.int32))
    # capacities nobody reaches change nothing; a single place in one expert
    big = [s.T * s.k] * s.N
    check_layer(s, inp, gpu_forward(s, inp, layer=L, cap=big), cap=np.array(big, np.int32))
    one = list(big)
    one[0] = 1
    r1 = gpu_forward(s, inp, layer=L, cap=one)
    check_layer(s, inp, r1, cap=np.array(one, np.int32))
    assert r1["kept"][0] == 1 and r1["counts"][0] > 1


def test_workload_mid_with_the_papers_capacity_sampled():
    """Ragged groups (router bias) at gamma = 1.1, tau = 0.75: the large groups are cut."""
    s = WORKLOADS["mid"]
    inp = make_inputs(s)
    L = make_layer(s)
    cap = L.capacity(s.T, 1.1, 0.75)
    assert cap == oracle.capacity(s, 1.1, 0.75).tolist()
    res = gpu_forward(s, inp, variant=2, layer=L, cap=cap, balance_tau=0.75)
    toks = sample_tokens(s, res["topk_idx"], 4096, seed=9)
    errs = check_layer(s, inp, res, tok_list=toks, cap=np.array(cap, np.int32), balance_tau=0.75)
    say("mid with capacity", errs, "kept", res["kept"].tolist())
    assert errs["dropped"] > 0


# ------------------------------------------------------------------ edge cases
@pytest.mark.parametrize("variant", [1, 0])
def test_edge_routing_patterns(variant):
    s = small_shape("edge", T=700, n_ffn=6)
    N, nf = s.N, s.n_ffn
    rng = np.random.default_rng(3)
    zc = np.arange(nf, N)
    patterns = {}
    # every slot on a zero-computation expert: R = 0, the GEMMs have nothing to do
    patterns["all_zc"] = np.stack([rng.permutation(zc)[:2] for _ in range(s.T)])
    # every slot on an FFN expert
    patterns["all_ffn"] = np.stack([rng.permutation(nf)[:2] for _ in range(s.T)])
    # expert 2 empty, expert 4 has exactly one row, expert 0 takes most tokens
    idx = np.stack([rng.permutation([0, 1, 3, 5] + zc.tolist())[:2] for _ in range(s.T)])
    idx[:, 0] = np.where(rng.random(s.T) < 0.7, 0, idx[:, 0])
    idx[:, 1] = np.where(idx[:, 1] == idx[:, 0], 1, idx[:, 1])
    idx[17] = [4, 0]
    patterns["empty_and_single"] = idx
    # zero + copy for every token: the layer is bypassed up to the gate weight
    patterns["zero_copy"] = np.tile(np.array([[nf + 1, nf]]), (s.T, 1))
    # one expert holds everything (one long group), second slot constant experts
    patterns["one_group"] = np.stack([np.full(s.T, 3), nf + 2 + (np.arange(s.T) % 2)], 1)
    for name, idx in patterns.items():
        say("edge pattern", name, "variant", variant)
        inp = forced_routing(s, idx.astype(np.int64))
        res = gpu_forward(s, inp, variant=variant)
        assert np.array_equal(res["topk_idx"], idx), name
        errs = check_layer(s, inp, res, max_near_ties=0)
        say(name, errs)
        if name == "all_zc":
            assert errs["R"] == 0
        if name == "empty_and_single":
            assert res["counts"][2] == 0 and res["counts"][4] == 1
        if name == "zero_copy":
            g = res["topk_w"][:, 0].astype(np.float64)
            assert rel_err(res["out"], g[:, None] * inp["x"]) <= TOL_OUT["bf16"]


@pytest.mark.parametrize("kw", [dict(T=1), dict(T=2, k=1), dict(T=63), dict(T=65),
                                dict(T=5, n_ffn=2, n_zero=1, n_copy=1, n_const=0, k=4)])
def test_tiny_token_counts(kw):
    s = small_shape("few", **kw)
    inp = make_inputs(s)
    say("few tokens", kw)
    for variant in (1, 0):
        res = gpu_forward(s, inp, variant=variant)
        check_layer(s, inp, res)


@pytest.mark.parametrize("act", ["bf16", "f32"])
@pytest.mark.parametrize("kw", [
    dict(T=1, seed=118),                         # one token
    dict(T=64, seed=119),                        # last size at which the router's second kernel also permutes
    dict(T=64, k=4, seed=120),                   # ... with four slots per token
    dict(T=65, seed=121),                        # first size with a permutation launch of its own
    dict(T=256, seed=111),                       # last size of the few-token router
    dict(T=257, seed=112),                       # first size of the ordinary routers
    dict(T=2048, seed=113),                      # 4096 slots: last size of the one-workgroup permutation
    dict(T=2049, seed=114),                      # first size of the three-kernel permutation
    dict(T=1366, k=3, seed=115),                 # 4098 slots
    dict(T=200, D=1000, F=64, n_ffn=3, seed=116),  # D not a multiple of the router's K tile
    dict(T=100, D=4160, F=64, n_ffn=3, seed=117),  # more K tiles than slices, ragged last slice
])
def test_few_token_kernels_and_their_size_limits(kw, act):
    """Calls on both sides of the sizes at which the library changes kernels,
    with expert capacities and load-balance statistics on."""
    s = small_shape("limits", act=act, **kw)
    inp = make_inputs(s)
    say("size limits", kw, act)
    L = make_layer(s)
    cap = L.capacity(s.T, 1.1, 0.75)
    res = gpu_forward(s, inp, layer=L, cap=cap, balance_tau=0.75)
    errs = check_layer(s, inp, res, cap=np.array(cap, np.int32), balance_tau=0.75)
    say("  ", errs)


def test_few_token_step_calls_with_capacities_set_after_the_routing():
    """At a handful of tokens the routing call already groups the slots.  Capacities
    set between moepp_route and moepp_permute must still take effect, a repeated
    moepp_permute must change nothing, and the step calls must give what one
    moepp_layer_forward call gives."""
    import torch
    s = small_shape("fewsteps", T=48, seed=131)
    inp = make_inputs(s)
    dev = to_device(s, inp)
    L = make_layer(s)
    cap = [max(1, c // 2) for c in L.capacity(s.T, 1.1, 0.75)]      # tight: assignments are dropped
    ref = gpu_forward(s, inp, layer=L, dev=dev, cap=cap)             # capacities first, one call
    assert int(ref["kept"].sum()) < s.T * s.k, "the capacities of this test must drop something"
    check_layer(s, inp, ref, cap=np.array(cap, np.int32))
    packed = L.pack_experts(dev["w1"], dev["w3"], dev["w2"])
    L.set_capacity(None)
    L.route(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], dev["W_c"])
    torch.cuda.synchronize()
    assert int(L.get_kept().sum().item()) == s.T * s.k               # grouped without capacities
    L.set_capacity(cap)
    for _ in range(2):
        L.permute()
        L.expert_ffn(dev["x"], packed)
        out = L.combine(dev["x"], dev["const_vecs"])
        torch.cuda.synchronize()
        r = L.get_routing()
        for key in ("counts", "offsets", "row_of"):
            assert np.array_equal(r[key].cpu().numpy(), ref[key]), key
        R = int(ref["offsets"][-1])
        assert np.array_equal(r["src_of"].cpu().numpy()[:R], ref["src_of"][:R])
        assert np.array_equal(L.get_kept().cpu().numpy(), ref["kept"])
        assert np.array_equal(out.float().cpu().numpy().astype(np.float64), ref["out"])


def test_zero_tokens_and_smaller_T_than_T_max():
    s = small_shape("tmax", T=200)
    inp = make_inputs(s)
    dev = to_device(s, inp)
    L = make_layer(s, T_max=512)
    res = gpu_forward(s, inp, layer=L, dev=dev)
    check_layer(s, inp, res)
    s0 = s.with_(T=0)
    res0 = gpu_forward(s0, inp, layer=L, dev=dev)
    assert res0["out"].shape == (0, s.D)
    # a shorter call on the same context afterwards
    s2 = s.with_(T=77)
    inp2 = {k: (v[:77] if k in ("x", "prev_gate") else v) for k, v in inp.items()}
    res2 = gpu_forward(s2, inp2, layer=L, dev=dev)
    check_layer(s2, inp2, res2)


def test_no_ffn_experts_layer():
    s = small_shape("zc_only", n_ffn=0, n_zero=1, n_copy=2, n_const=2, T=150)
    inp = make_inputs(s)
    res = gpu_forward(s, inp)
    check_layer(s, inp, res)


def test_two_runs_are_bytewise_identical():
    import torch
    s = small_shape("determinism", T=1500, D=512, F=384)
    inp = make_inputs(s)
    dev = to_device(s, inp)
    L = make_layer(s)
    packed = L.pack_experts(dev["w1"], dev["w3"], dev["w2"])
    outs = []
    for _ in range(2):
        out, gate = L.layer_forward(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], packed,
                                    dev["const_vecs"], dev["W_c"])
        torch.cuda.synchronize()
        r = L.get_routing()
        outs.append([out.clone(), gate.clone()] + [r[k].clone() for k in sorted(r)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_step_calls_equal_the_fused_call_and_timing_reports():
    import torch
    s = small_shape("steps", T=2304, D=256, F=256)        # enough slots for the three-kernel permutation
    inp = make_inputs(s)
    dev = to_device(s, inp)
    L = make_layer(s)
    packed = L.pack_experts(dev["w1"], dev["w3"], dev["w2"])
    out, gate = L.layer_forward(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], packed,
                                dev["const_vecs"], dev["W_c"])
    torch.cuda.synchronize()
    out = out.clone()
    L.set_timing(True)
    gate2 = L.route(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], dev["W_c"])
    L.permute()
    L.expert_ffn(dev["x"], packed)
    out2 = L.combine(dev["x"], dev["const_vecs"])
    torch.cuda.synchronize()
    assert torch.equal(out, out2) and torch.equal(gate, gate2)
    L.layer_forward(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], packed,
                    dev["const_vecs"], dev["W_c"])
    ms = L.get_timing()
    say("kernel ms", ms)
    # the router kernel counts its own selections and the scatter kernel scans: no
    # histogram or scan kernel of their own at this size; the statistics are off
    assert all(v > 0 for k, v in ms.items() if k not in ("balance", "perm_hist", "perm_scan"))
    assert ms["balance"] == 0 and ms["perm_hist"] == 0 and ms["perm_scan"] == 0
    L.set_variant(1)                                  # the generic router leaves no histogram
    L.layer_forward(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], packed,
                    dev["const_vecs"], dev["W_c"])
    ms = L.get_timing()
    assert ms["perm_hist"] > 0 and ms["perm_scatter"] > 0
    L.set_timing(False)


@pytest.mark.parametrize("variant", [1, 2])
def test_more_chunks_than_one_scatter_kernel_scans_itself(variant):
    """So many slots that the permutation falls back to a scan kernel of its own
    (more than 2048 chunks), with capacities and load-balance statistics on; with
    the MFMA router the chunks are the router's 64-token workgroups (more of them
    than the statistics have rows for: the pass over the logits runs), with the
    generic one 256 slots."""
    s = small_shape("manychunks", T=270000, D=128, F=64, n_ffn=5, seed=151)
    inp = make_inputs(s)
    L = make_layer(s)
    cap = L.capacity(s.T, 1.1, 0.75)
    res = gpu_forward(s, inp, variant=variant, layer=L, cap=cap, intermediates=False, balance_tau=0.75)
    toks = sample_tokens(s, res["topk_idx"], 2048, seed=3)
    say("many chunks", check_layer(s, inp, res, tok_list=toks, cap=np.array(cap, np.int32), check_inter=False,
                                   balance_tau=0.75))


def test_step_calls_in_any_mix_leave_the_same_permutation():
    """moepp_permute after moepp_route (the router's own histogram), a second
    moepp_permute without a new route (its own histogram pass), and with other
    capacities in between: the tables are always those of the oracle."""
    import torch
    s = small_shape("mix", T=6000, D=256, F=128, n_ffn=6, seed=161)
    inp = make_inputs(s)
    dev = to_device(s, inp)
    L = make_layer(s)
    L.set_variant(2)
    ref = oracle.permute(s, oracle.route(s, inp["x"], inp["prev_gate"], inp["W_g"], inp["W_res"])["topk_idx"])
    L.route(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], dev["W_c"])
    for rep in range(3):
        if rep == 1:
            L.set_capacity([7] * s.N)
        if rep == 2:
            L.set_capacity(None)
        L.permute()
        torch.cuda.synchronize()
        r = {k: v.cpu().numpy() for k, v in L.get_routing().items()}
        if rep == 1:
            assert r["offsets"][-1] == 7 * s.n_ffn and (r["row_of"] == -2).sum() > 0
            continue
        if not np.array_equal(r["topk_idx"], oracle.route(s, inp["x"], inp["prev_gate"], inp["W_g"],
                                                           inp["W_res"])["topk_idx"]):
            pytest.skip("a near-tie token in this seed")
        for k in ("counts", "offsets", "row_of"):
            assert np.array_equal(r[k], ref[k]), (rep, k)
        R = int(ref["offsets"][-1])
        assert np.array_equal(r["src_of"][:R], ref["src_of"][:R]), rep


@pytest.mark.parametrize("kw", [
    dict(T=40, D=512, F=768, n_ffn=6, seed=171),          # K = 512 / 768: 2 and 3 steps per wave
    dict(T=64, D=1024, F=256, n_ffn=8, seed=172),
    dict(T=7, D=256, F=512, n_ffn=3, k=3, seed=173),
    dict(T=30, D=1280, F=1536, n_ffn=4, seed=174),        # 5 and 6 steps per wave
])
def test_few_rows_per_expert_take_the_weight_streaming_kernels(kw):
    """T * k <= 16 n_ffn: the FFN runs in the kernels that only stream the expert
    weights.  Checked against the oracle, and against the tiled kernels (variant 3)."""
    s = small_shape("decode", **kw)
    assert s.T * s.k <= 16 * s.n_ffn and s.D % 256 == 0 and s.F % 256 == 0
    inp = make_inputs(s)
    say("decode", kw)
    a = gpu_forward(s, inp, variant=2)
    say("errs", check_layer(s, inp, a))
    b = gpu_forward(s, inp, variant=3)
    assert np.array_equal(a["topk_idx"], b["topk_idx"]) and np.array_equal(a["row_of"], b["row_of"])
    assert rel_err(a["h"], b["h"]) <= 1e-2 and rel_err(a["out"], b["out"]) <= 1e-2


def test_weight_streaming_kernels_with_long_empty_and_single_row_groups():
    """Forced routing: one expert takes 37 rows (three blocks of 16, the last with
    5 rows), one takes none (its weights must not be needed), one takes a single row."""
    s = small_shape("decode_groups", T=48, D=512, F=512, n_ffn=6, seed=175)
    nf = s.n_ffn
    idx = np.empty((s.T, 2), np.int64)
    idx[:, 0] = np.where(np.arange(s.T) < 37, 1, 3)            # expert 1: 37 rows, expert 3: 11 rows
    idx[:, 1] = nf + (np.arange(s.T) % (s.N - nf))              # zero-computation experts
    idx[40, 1] = 4                                              # expert 4: one row; experts 0, 2, 5: none
    inp = forced_routing(s, idx)
    # poison the weights of the experts without rows: a kernel that touched them would show it
    for name in ("w1", "w3", "w2"):
        for e in (0, 2, 5):
            inp[name][e] = np.float32(np.nan)
    res = gpu_forward(s, inp, variant=2)
    assert np.array_equal(res["topk_idx"], idx)
    assert res["counts"][:nf].tolist() == [0, 37, 0, 11, 1, 0]
    assert np.isfinite(res["out"]).all()
    inp_ok = {k: (np.nan_to_num(v) if k in ("w1", "w3", "w2") else v) for k, v in inp.items()}
    say("errs", check_layer(s, inp_ok, res, max_near_ties=0))


def test_mfma_and_generic_kernels_agree():
    """The two kernel families must give the same routing and close outputs."""
    s = small_shape("families", T=900, D=512, F=768, n_ffn=6)
    inp = make_inputs(s)
    a = gpu_forward(s, inp, variant=1)
    b = gpu_forward(s, inp, variant=2)
    assert rel_err(b["out_gate"], a["out_gate"]) <= 1e-5
    same = (a["topk_idx"] == b["topk_idx"]).all(axis=1)
    assert same.mean() > 0.995
    assert rel_err(b["out"][same], a["out"][same]) <= 1e-2


def test_gemm_tail_launch_is_bitwise_the_single_launch():
    """A problem of a few rounds of tiles whose last round is sparsely filled is
    finished by a second launch with half-height tiles: same bits as one launch,
    and right against the oracle."""
    s = small_shape("tail", T=9000, D=512, F=1024, n_ffn=5, seed=131)
    inp = make_inputs(s)
    a = gpu_forward(s, inp, variant=3)               # the default geometry without the tail launch
    b = gpu_forward(s, inp, variant=2)
    m_tiles = int(sum(-(-int(c) // 256) for c in b["counts"][:s.n_ffn]))
    left1, left2 = m_tiles * (2 * s.F // 256) % 256, m_tiles * (s.D // 256) % 256
    say("tail: m tiles", m_tiles, "leftover tiles GEMM1", left1, "GEMM2", left2)
    assert 0 < left1 <= 128 and 0 < left2 <= 128     # both GEMMs take the tail path (256 workgroups)
    for k in ("out", "yffn", "h", "topk_idx", "row_of"):
        assert np.array_equal(a[k], b[k]), k
    check_layer(s, inp, b)


# ------------------------------------------------- the benchmark's own shapes
def _full_size(name, n_sample, check_inter=True, capacity=None):
    """One forward of a benchmark workload with the kernels bench.py times
    (variant 2: the MFMA kernels must cover every benchmark shape), compared
    with the oracle: routing, counts and the permutation on all tokens, out / h /
    yffn on all tokens (n_sample None) or on a seeded sample that covers every
    selected expert.  capacity = (gamma, tau): Eq.8 capacities and Eq.7 statistics on."""
    s = WORKLOADS[name]
    say("workload", name, s)
    inp = make_inputs(s)
    say("inputs ready")
    L = make_layer(s)
    cap, tau = None, 0.0
    if capacity:
        cap = L.capacity(s.T, capacity[0], capacity[1])
        assert cap == oracle.capacity(s, capacity[0], capacity[1]).tolist()
        tau = capacity[1]
    res = gpu_forward(s, inp, variant=2, layer=L, cap=cap, balance_tau=tau,
                      intermediates=check_inter)
    say("gpu done, R =", int(res["offsets"][-1]), "counts", res["counts"].tolist(),
        "kept", res["kept"].tolist())
    toks = None if n_sample is None else sample_tokens(s, res["topk_idx"], n_sample, seed=s.seed)
    errs = check_layer(s, inp, res, tok_list=toks, check_inter=check_inter,
                       cap=None if cap is None else np.array(cap, np.int32), balance_tau=tau)
    say(name, "errs", errs)
    return s, res, errs


def test_workload_small_all_tokens():
    s, res, errs = _full_size("small", None)
    assert abs(errs["R"] / (s.T * s.k) - s.n_ffn / s.N) < 0.01      # Tab.1 with tau = 1


def test_workload_mid_ragged_groups_all_tokens():
    s, res, errs = _full_size("mid", None)
    c = res["counts"][:s.n_ffn]
    assert c.max() > 8 * max(c.min(), 1)


def test_workload_skew_all_tokens():
    s, res, errs = _full_size("skew", None)
    c = res["counts"].astype(np.float64)
    assert abs(c[s.n_ffn:].sum() / c.sum() - 0.5) < 0.03
    assert abs(c[0] / c[1:s.n_ffn].mean() - 4.0) < 0.5


def test_workload_smallbatch_all_tokens():
    _full_size("smallbatch", None)


def test_workload_large_sampled():
    s, res, errs = _full_size("large", 4096)
    assert abs(errs["R"] / (s.T * s.k) - s.n_ffn / s.N) < 0.01


def test_workload_large_with_the_papers_capacity_sampled():
    """The large layer as bench.py times it a second time: capacities of Eq.8 at
    gamma = 1.1, tau = 0.75 and the statistics of Eq.7 on."""
    s, res, errs = _full_size("large", 4096, capacity=(1.1, 0.75))
    assert errs["dropped"] > 0 and np.all(res["kept"] <= res["counts"])


def test_workload_large_two_kernel_families_all_tokens():
    """Every token of the benchmark workload through both kernel families (plain
    fp32 FMA kernels and the MFMA kernels): same routing except inside float32
    noise, outputs within the bf16 tolerance.  A consistency check between two
    HIP paths over all 32768 tokens; the oracle comparison is the sampled test above."""
    s = WORKLOADS["large"]
    inp = make_inputs(s)
    L = make_layer(s)
    dev = to_device(s, inp)
    a = gpu_forward(s, inp, variant=1, layer=L, dev=dev, intermediates=False)
    b = gpu_forward(s, inp, variant=2, layer=L, dev=dev, intermediates=False)
    assert rel_err(b["out_gate"], a["out_gate"]) <= 1e-5
    same = (a["topk_idx"] == b["topk_idx"]).all(axis=1)
    say("large, both families: tokens routed alike", int(same.sum()), "of", s.T)
    assert same.mean() > 0.999
    assert rel_err(b["out"][same], a["out"][same]) <= 1e-2
    assert rel_err(b["topk_w"][same], a["topk_w"][same]) <= 1e-5


@pytest.mark.parametrize("name", ["large_vanilla20", "large_vanilla16"])
def test_workload_large_vanilla_sampled(name):
    """The vanilla comparison layers of the benchmark (20 or 16 FFN experts, none other)."""
    s, res, errs = _full_size(name, 4096)
    assert errs["R"] == s.T * s.k
