"""Shared plumbing of the GPU parity tests: move seeded inputs to the device,
run the HIP path through the C ABI, compare with the CPU oracle.

Tolerances (stated where they are used):
  integer outputs (topk_idx, counts, offsets, row_of, src_of): bit-exact;
  out:       max|err| / max|ref| <= 1e-2 for bf16 layers, 1e-5 for fp32 layers;
  out_gate, topk_w, alpha1: max|err| / max|ref| <= 1e-5 (fp32 in every layer).
A token whose oracle logits have a gap <= 1e-4 around the Top-K boundary (or
between selected slots) may legally be routed differently by fp32 arithmetic
in another summation order; for those the oracle is re-run with the GPU's
selection forced, after checking that the GPU's choice is within the margin.
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2410_07348_amd.torch_util import make_layer, to_device  # noqa: F401  (re-exported)

MARGIN = 1e-4
TOL_OUT = {"bf16": 1e-2, "f32": 1e-5}
TOL_F32 = 1e-5


def gpu_forward(shape, inp, variant=0, layer=None, dev=None, intermediates=True, cap=None,
                balance_tau=0.0):
    """One moepp_layer_forward call; every output copied back as numpy.
    cap: per-expert capacities (None: unlimited); balance_tau > 0: also the
    load-balance statistics of Eq.7."""
    import torch
    dev = dev or to_device(shape, inp)
    L = layer or make_layer(shape)
    L.set_variant(variant)
    L.set_capacity(cap)
    L.set_balance(balance_tau)
    packed = L.pack_experts(dev["w1"], dev["w3"], dev["w2"]) if shape.n_ffn else None
    L.set_router_bias(dev.get("bias"))
    cv = dev["const_vecs"] if shape.n_const else None
    wc = dev["W_c"] if shape.n_const else None
    x = dev["x"][:shape.T]
    pg = dev["prev_gate"][:shape.T] if dev.get("prev_gate") is not None else None
    out, out_gate = L.layer_forward(x, pg, dev["W_g"], dev.get("W_res"), packed, cv, wc,
                                    k=shape.k)
    torch.cuda.synchronize()
    res = {"out": out.float().cpu().numpy().astype(np.float64),
           "out_gate": out_gate.cpu().numpy()}
    if shape.T == 0:
        return res
    for k, v in L.get_routing().items():
        res[k] = v.cpu().numpy().copy()
    res["kept"] = L.get_kept().cpu().numpy().copy()
    if balance_tau > 0:
        for k, v in L.get_balance().items():
            res[k] = v.cpu().numpy().astype(np.float64)
    if intermediates:
        R = int(res["offsets"][-1]) if shape.n_ffn else 0
        for k, v in L.get_intermediates(R).items():
            res[k] = v.float().cpu().numpy()
    return res


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def reconcile_routing(shape, inp, res):
    """Oracle routing, re-run with the GPU's selection forced where the two
    differ inside the margin.  Returns (oracle routing dict, n_near_tie)."""
    r = oracle.route(shape, inp["x"], inp.get("prev_gate"), inp["W_g"], inp.get("W_res"),
                     inp.get("bias"), want_probs=True)
    diff = np.nonzero((r["topk_idx"] != res["topk_idx"]).any(axis=1))[0]
    if diff.size:
        L = r["out_gate"].astype(np.float64)
        for t in diff:
            kth = np.sort(L[t])[::-1][shape.k - 1]
            sel = res["topk_idx"][t]
            assert len(set(sel.tolist())) == shape.k, "token %d: repeated expert %s" % (t, sel)
            assert np.all(L[t, sel] >= kth - MARGIN), \
                "token %d: GPU selected %s outside the %g margin (oracle %s, logits %s)" % (
                    t, sel, MARGIN, r["topk_idx"][t], L[t])
            # slot order must be descending up to the margin
            assert np.all(np.diff(L[t, sel]) <= MARGIN), "token %d: slot order" % t
        r = oracle.route(shape, inp["x"], inp.get("prev_gate"), inp["W_g"], inp.get("W_res"),
                         inp.get("bias"), forced_idx=res["topk_idx"], want_probs=True)
    return r, int(diff.size)


def check_layer(shape, inp, res, tok_list=None, max_near_ties=None, check_inter=True, cap=None,
                balance_tau=0.0):
    """Compare one GPU forward with the oracle.  Returns a dict of measured
    errors (for reporting).  cap / balance_tau as given to gpu_forward."""
    s = shape
    r, near = reconcile_routing(s, inp, res)
    if max_near_ties is None:
        max_near_ties = max(2, s.T // 500)
    assert near <= max_near_ties, "%d tokens routed differently (near ties)" % near
    # routing: bit-exact indices
    assert np.array_equal(res["topk_idx"], r["topk_idx"])
    e_gate = rel_err(res["out_gate"], r["out_gate"])
    e_w = rel_err(res["topk_w"], r["topk_w"])
    assert e_gate <= TOL_F32, "out_gate rel err %g" % e_gate
    assert e_w <= TOL_F32, "topk_w rel err %g" % e_w
    # permutation: bit-exact
    if cap is None:
        p = oracle.permute(s, r["topk_idx"])
        p["kept"] = p["counts"]
        row_of = None
    else:
        p = oracle.permute_capacity(s, r["topk_idx"], cap)
        row_of = p["row_of"]
    R = int(p["offsets"][-1])
    assert np.array_equal(res["kept"], p["kept"])
    assert np.array_equal(res["counts"], p["counts"])
    assert np.array_equal(res["offsets"], p["offsets"])
    assert np.array_equal(res["row_of"], p["row_of"])
    assert np.array_equal(res["src_of"][:R], p["src_of"][:R])
    assert int(res["counts"].sum()) == s.T * s.k
    # outputs
    want = dict(want_slots=check_inter, want_h=check_inter, want_alpha=True)
    o = oracle.experts(s, inp["x"], r["topk_idx"], r["topk_w"], inp["w1"], inp["w3"],
                       inp["w2"], inp["const_vecs"], inp["W_c"], tok_list=tok_list,
                       row_of=row_of, **want)
    toks = np.arange(s.T) if tok_list is None else np.asarray(tok_list)
    e_out = rel_err(res["out"][toks], o["out"])
    assert e_out <= TOL_OUT[s.act], "out rel err %g > %g" % (e_out, TOL_OUT[s.act])
    errs = {"out": e_out, "out_gate": e_gate, "topk_w": e_w, "near_ties": near, "R": R,
            "dropped": int(s.T * s.k - p["kept"].sum())}
    if balance_tau > 0:
        b = oracle.balance(s, r["probs"], r["topk_idx"], balance_tau)
        assert np.array_equal(res["f"], b["f"].astype(np.float32))      # counts / T, one rounding
        errs["P"] = rel_err(res["P"], b["P"])
        errs["loss"] = abs(float(res["loss"][0]) - b["loss"]) / abs(b["loss"])
        assert errs["P"] <= TOL_F32 and errs["loss"] <= TOL_F32, errs
    if s.n_const and "alpha1" in res:
        e_a = rel_err(res["alpha1"][toks], o["alpha1"])
        assert e_a <= TOL_F32, "alpha1 rel err %g" % e_a
        errs["alpha1"] = e_a
    if check_inter and s.n_ffn and R and "h" in res:
        # per-kernel parity of the grouped FFN: rows of the sampled tokens
        rows, hh, yy = [], [], []
        for u, t in enumerate(toks):
            for sl in range(s.k):
                row = p["row_of"][t * s.k + sl]
                if row >= 0:
                    rows.append(row)
                    hh.append(o["h"][u, sl])
                    yy.append(o["slot_out"][u, sl])
        if rows:
            rows = np.asarray(rows)
            errs["h"] = rel_err(res["h"][rows], np.asarray(hh))
            errs["yffn"] = rel_err(res["yffn"][rows], np.asarray(yy))
            assert errs["h"] <= TOL_OUT[s.act], "h rel err %g" % errs["h"]
            assert errs["yffn"] <= TOL_OUT[s.act], "yffn rel err %g" % errs["yffn"]
    return errs


def sample_tokens(shape, res_topk_idx, n, seed=0):
    """Seeded sample of n tokens that covers every selected expert at least
    once (when the routing uses it at all)."""
    rng = np.random.default_rng(seed)
    T = shape.T
    chosen = set(rng.choice(T, size=min(n, T), replace=False).tolist())
    N = shape.n_ffn + shape.n_zero + shape.n_copy + shape.n_const
    for e in range(N):
        hit = np.nonzero((res_topk_idx == e).any(axis=1))[0]
        if hit.size:
            chosen.add(int(hit[0]))
    return np.array(sorted(chosen), dtype=np.int32)
