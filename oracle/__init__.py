"""ctypes front end of the CPU oracle (oracle/moepp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg; never by the HIP package.  This wrapper only
marshals numpy arrays; all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moepp_oracle.c")
_LIB = os.path.join(_HERE, "libmoepp_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over tokens only)."""
    if (force or not os.path.exists(_LIB)
            or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC",
                               "-shared", "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("T", "D", "F", "n_ffn", "n_zero", "n_copy", "n_const", "k")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.moepp_oracle_threads.restype = ctypes.c_int
        for f in ("moepp_oracle_route", "moepp_oracle_permute",
                  "moepp_oracle_experts", "moepp_oracle_dense",
                  "moepp_oracle_capacity", "moepp_oracle_permute_capacity",
                  "moepp_oracle_balance"):
            getattr(_lib, f).restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(lib().moepp_oracle_threads())


def _cshape(T, D, F, n_ffn, n_zero, n_copy, n_const, k):
    return _Shape(T, D, F, n_ffn, n_zero, n_copy, n_const, k)


def _p(a, dtype):
    """Pointer to a C-contiguous numpy array of the given dtype (or NULL)."""
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, \
        (type(a), getattr(a, "dtype", None), dtype)
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def route(sh, x, prev_gate, W_g, W_res, bias=None, forced_idx=None,
          want_probs=False):
    """Eq.2/Eq.6 router, softmax and Top-K (Eq.1) for all tokens.
    `sh` is any object with T, D, F, n_ffn, n_zero, n_copy, n_const, k."""
    cs = _cshape(sh.T, sh.D, sh.F, sh.n_ffn, sh.n_zero, sh.n_copy, sh.n_const, sh.k)
    N = sh.n_ffn + sh.n_zero + sh.n_copy + sh.n_const
    x, prev_gate, W_g, W_res, bias = map(_f32, (x, prev_gate, W_g, W_res, bias))
    assert x.shape == (sh.T, sh.D) and W_g.shape == (N, sh.D)
    if (prev_gate is None) != (W_res is None):
        raise ValueError("prev_gate and W_res are given together or not at all")
    if prev_gate is not None:
        assert prev_gate.shape == (sh.T, N) and W_res.shape == (N, N)
    if forced_idx is not None:
        forced_idx = np.ascontiguousarray(forced_idx, dtype=np.int32)
        assert forced_idx.shape == (sh.T, sh.k)
    out_gate = np.empty((sh.T, N), np.float32)
    probs = np.empty((sh.T, N), np.float64) if want_probs else None
    idx = np.empty((sh.T, sh.k), np.int32)
    w = np.empty((sh.T, sh.k), np.float32)
    rc = lib().moepp_oracle_route(ctypes.byref(cs), _p(x, np.float32),
                                  _p(prev_gate, np.float32), _p(W_g, np.float32),
                                  _p(W_res, np.float32), _p(bias, np.float32),
                                  _p(forced_idx, np.int32), _p(out_gate, np.float32),
                                  _p(probs, np.float64), _p(idx, np.int32),
                                  _p(w, np.float32))
    if rc != 0:
        raise ValueError("moepp_oracle_route: invalid shape")
    r = {"out_gate": out_gate, "topk_idx": idx, "topk_w": w}
    if want_probs:
        r["probs"] = probs
    return r


def permute(sh, topk_idx):
    """counts / offsets / row_of / src_of of the grouping by FFN expert."""
    cs = _cshape(sh.T, sh.D, sh.F, sh.n_ffn, sh.n_zero, sh.n_copy, sh.n_const, sh.k)
    N = sh.n_ffn + sh.n_zero + sh.n_copy + sh.n_const
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    assert idx.shape == (sh.T, sh.k)
    counts = np.empty(N, np.int32)
    offsets = np.empty(sh.n_ffn + 1, np.int32)
    row_of = np.empty(sh.T * sh.k, np.int32)
    src_of = np.empty(sh.T * sh.k, np.int32)
    rc = lib().moepp_oracle_permute(ctypes.byref(cs), _p(idx, np.int32),
                                    _p(counts, np.int32), _p(offsets, np.int32),
                                    _p(row_of, np.int32), _p(src_of, np.int32))
    if rc != 0:
        raise ValueError("moepp_oracle_permute: expert index out of range")
    return {"counts": counts, "offsets": offsets, "row_of": row_of, "src_of": src_of}


def capacity(sh, gamma, tau, per_assignment=True):
    """Expert capacities C_i of Eq.8 (int32 [N]): for T*K assignments, or with
    per_assignment=False for T tokens, the equation as it is printed."""
    cs = _cshape(sh.T, sh.D, sh.F, sh.n_ffn, sh.n_zero, sh.n_copy, sh.n_const, sh.k)
    N = sh.n_ffn + sh.n_zero + sh.n_copy + sh.n_const
    cap = np.empty(N, np.int32)
    rc = lib().moepp_oracle_capacity(ctypes.byref(cs), ctypes.c_double(gamma),
                                     ctypes.c_double(tau), ctypes.c_int32(1 if per_assignment else 0),
                                     _p(cap, np.int32))
    if rc != 0:
        raise ValueError("moepp_oracle_capacity: gamma and tau must be positive")
    return cap


def permute_capacity(sh, topk_idx, cap):
    """Grouping in which expert i keeps its first cap[i] assignments."""
    cs = _cshape(sh.T, sh.D, sh.F, sh.n_ffn, sh.n_zero, sh.n_copy, sh.n_const, sh.k)
    N = sh.n_ffn + sh.n_zero + sh.n_copy + sh.n_const
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    cap = np.ascontiguousarray(cap, dtype=np.int32)
    assert idx.shape == (sh.T, sh.k) and cap.shape == (N,)
    counts = np.empty(N, np.int32)
    kept = np.empty(N, np.int32)
    offsets = np.empty(sh.n_ffn + 1, np.int32)
    row_of = np.empty(sh.T * sh.k, np.int32)
    src_of = np.empty(sh.T * sh.k, np.int32)
    rc = lib().moepp_oracle_permute_capacity(ctypes.byref(cs), _p(idx, np.int32),
                                             _p(cap, np.int32), _p(counts, np.int32),
                                             _p(kept, np.int32), _p(offsets, np.int32),
                                             _p(row_of, np.int32), _p(src_of, np.int32))
    if rc != 0:
        raise ValueError("moepp_oracle_permute_capacity: bad expert index or capacity")
    return {"counts": counts, "kept": kept, "offsets": offsets, "row_of": row_of,
            "src_of": src_of}


def balance(sh, probs, topk_idx, tau):
    """f_i, P_i and the heterogeneous load-balance loss L_b of Eq.7."""
    cs = _cshape(sh.T, sh.D, sh.F, sh.n_ffn, sh.n_zero, sh.n_copy, sh.n_const, sh.k)
    N = sh.n_ffn + sh.n_zero + sh.n_copy + sh.n_const
    probs = np.ascontiguousarray(probs, dtype=np.float64)
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    assert probs.shape == (sh.T, N) and idx.shape == (sh.T, sh.k)
    f = np.empty(N, np.float64)
    P = np.empty(N, np.float64)
    loss = np.empty(1, np.float64)
    rc = lib().moepp_oracle_balance(ctypes.byref(cs), _p(probs, np.float64),
                                    _p(idx, np.int32), ctypes.c_double(tau),
                                    _p(f, np.float64), _p(P, np.float64),
                                    _p(loss, np.float64))
    if rc != 0:
        raise ValueError("moepp_oracle_balance: needs at least one token")
    return {"f": f, "P": P, "loss": float(loss[0])}


def experts(sh, x, topk_idx, topk_w, w1, w3, w2, const_vecs, W_c, tok_list=None,
            want_slots=False, want_h=False, want_alpha=False, row_of=None):
    """Selected experts (Eq.2-5) and their weighted sum (Eq.1) per token;
    assignments with row_of == -2 (dropped by the capacity) are left out."""
    cs = _cshape(sh.T, sh.D, sh.F, sh.n_ffn, sh.n_zero, sh.n_copy, sh.n_const, sh.k)
    x, w1, w3, w2, const_vecs, W_c = map(_f32, (x, w1, w3, w2, const_vecs, W_c))
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    w = np.ascontiguousarray(topk_w, dtype=np.float32)
    assert x.shape == (sh.T, sh.D) and idx.shape == (sh.T, sh.k) == w.shape
    assert w1.shape == (sh.n_ffn, sh.F, sh.D) == w3.shape
    assert w2.shape == (sh.n_ffn, sh.D, sh.F)
    assert const_vecs.shape == (sh.n_const, sh.D) and W_c.shape == (sh.n_const, 2, sh.D)
    if tok_list is None:
        n_tok, tl = sh.T, None
    else:
        tl = np.ascontiguousarray(tok_list, dtype=np.int32)
        n_tok = int(tl.size)
    if row_of is not None:
        row_of = np.ascontiguousarray(row_of, dtype=np.int32)
        assert row_of.shape == (sh.T * sh.k,)
    out = np.empty((n_tok, sh.D), np.float64)
    slots = np.zeros((n_tok, sh.k, sh.D), np.float64) if want_slots else None
    h = np.zeros((n_tok, sh.k, sh.F), np.float64) if want_h else None
    a1 = np.zeros((n_tok, sh.n_const), np.float64) if want_alpha else None
    rc = lib().moepp_oracle_experts(ctypes.byref(cs), _p(x, np.float32),
                                    _p(idx, np.int32), _p(w, np.float32),
                                    _p(w1, np.float32), _p(w3, np.float32),
                                    _p(w2, np.float32), _p(const_vecs, np.float32),
                                    _p(W_c, np.float32), _p(row_of, np.int32),
                                    ctypes.c_int32(n_tok),
                                    _p(tl, np.int32), _p(out, np.float64),
                                    _p(slots, np.float64), _p(h, np.float64),
                                    _p(a1, np.float64))
    if rc != 0:
        raise ValueError("moepp_oracle_experts: token index out of range")
    r = {"out": out}
    if want_slots:
        r["slot_out"] = slots
    if want_h:
        r["h"] = h
    if want_alpha:
        r["alpha1"] = a1
    return r


def dense(sh, x, gate, w1, w3, w2, const_vecs, W_c):
    """Eq.1 literally: all N experts on every token, summed with gate [T,N]."""
    cs = _cshape(sh.T, sh.D, sh.F, sh.n_ffn, sh.n_zero, sh.n_copy, sh.n_const, sh.k)
    x, w1, w3, w2, const_vecs, W_c = map(_f32, (x, w1, w3, w2, const_vecs, W_c))
    gate = np.ascontiguousarray(gate, dtype=np.float64)
    out = np.empty((sh.T, sh.D), np.float64)
    lib().moepp_oracle_dense(ctypes.byref(cs), _p(x, np.float32), _p(gate, np.float64),
                             _p(w1, np.float32), _p(w3, np.float32),
                             _p(w2, np.float32), _p(const_vecs, np.float32),
                             _p(W_c, np.float32), _p(out, np.float64))
    return out


def layer_forward(sh, inp, forced_idx=None, tok_list=None, cap=None, **want):
    """Whole layer: route -> permute -> experts.  `inp` is a dict with the
    tensor names of workloads.make_inputs; `cap` [N] are expert capacities
    (None: unlimited)."""
    r = route(sh, inp["x"], inp.get("prev_gate"), inp["W_g"], inp.get("W_res"),
              inp.get("bias"), forced_idx=forced_idx, want_probs=True)
    if cap is None:
        r.update(permute(sh, r["topk_idx"]))
        row_of = None
    else:
        r.update(permute_capacity(sh, r["topk_idx"], cap))
        row_of = r["row_of"]
    r.update(experts(sh, inp["x"], r["topk_idx"], r["topk_w"], inp["w1"], inp["w3"],
                     inp["w2"], inp["const_vecs"], inp["W_c"], tok_list=tok_list,
                     row_of=row_of, **want))
    return r
