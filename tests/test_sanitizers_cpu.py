"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host code: the
CPU oracle, and the host side of libmoepp.so (validation, workspace layout,
Eq.8 arithmetic).  Each is driven by a small C program under tests/sanitize/;
a sanitizer report aborts the program, which fails the test.  The oracle's
driver prints checksums of every output, which must equal the ones the
ordinary -O2 build gives on the same seeded inputs.  No GPU is needed: the
device code of the library is compiled as usual but never launched."""
import os
import subprocess
from types import SimpleNamespace as NS

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-4000:], r.stderr[-4000:])
    return r.stdout


class Lcg:
    """The generator of tests/sanitize/oracle_main.c."""

    def __init__(self, seed):
        self.s = seed

    def fill(self, n, scale):
        out = np.empty(n, np.float32)
        s = self.s
        for i in range(n):
            s = (s * 6364136223846793005 + 1442695040888963407) & 0xFFFFFFFFFFFFFFFF
            out[i] = np.float32(scale) * np.float32((s >> 40) / 8388608.0 - 1.0)
        self.s = s
        return out


def checksum(a):
    a = np.asarray(a).reshape(-1)
    wts = 1 + np.arange(a.size) % 7
    if a.dtype.kind == "i":
        return int((a.astype(np.int64) * wts).sum())
    s = 0.0
    for v, w_ in zip(a.astype(np.float64).tolist(), wts.tolist()):     # the driver's summation order
        s += v * w_
    return s


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-std=c11", "-g", "-O1", "-fopenmp", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-static-libasan",
         "-static-libubsan", "-Wall", os.path.join(ROOT, "oracle", "moepp_oracle.c"),
         os.path.join(SAN, "oracle_main.c"), "-o", exe, "-lm"])
    got = {}
    for line in run([exe], env=ENV).splitlines():
        k, v = line.split()
        got[k] = float(v)
    assert got["status"] == 0 and got["experts.bad_token"] == -1

    # the same calls through the ordinary build
    s = NS(T=37, D=24, F=16, n_ffn=5, n_zero=1, n_copy=1, n_const=2, k=3)
    N, g = 9, Lcg(20241007)
    x = g.fill(s.T * s.D, 1.0).reshape(s.T, s.D)
    prev = g.fill(s.T * N, 1.0).reshape(s.T, N)
    W_g = g.fill(N * s.D, 0.2).reshape(N, s.D)
    W_res = g.fill(N * N, 0.2).reshape(N, N)
    bias = g.fill(N, 0.5)
    w1 = g.fill(s.n_ffn * s.F * s.D, 0.2).reshape(s.n_ffn, s.F, s.D)
    w3 = g.fill(s.n_ffn * s.F * s.D, 0.2).reshape(s.n_ffn, s.F, s.D)
    w2 = g.fill(s.n_ffn * s.D * s.F, 0.2).reshape(s.n_ffn, s.D, s.F)
    cv = g.fill(s.n_const * s.D, 0.2).reshape(s.n_const, s.D)
    W_c = g.fill(s.n_const * 2 * s.D, 0.2).reshape(s.n_const, 2, s.D)
    bias[2] = -100.0
    want = {}
    r = oracle.route(s, x, prev, W_g, W_res, bias, want_probs=True)
    for k in ("out_gate", "probs", "topk_idx", "topk_w"):
        want["route." + k] = checksum(r[k])
    assert 2 not in r["topk_idx"]
    r1 = oracle.route(s, x, None, W_g, None)
    want["first.out_gate"], want["first.topk_idx"] = checksum(r1["out_gate"]), checksum(r1["topk_idx"])
    rf = oracle.route(s, x, prev, W_g, W_res, bias, forced_idx=r1["topk_idx"])
    want["forced.topk_idx"], want["forced.topk_w"] = checksum(rf["topk_idx"]), checksum(rf["topk_w"])
    p = oracle.permute(s, r["topk_idx"])
    R = int(p["offsets"][-1])
    for k in ("counts", "offsets", "row_of"):
        want["permute." + k] = checksum(p[k])
    want["permute.src_of"] = checksum(p["src_of"][:R])
    want["capacity.assignments"] = checksum(oracle.capacity(s, 1.1, 0.75))
    cap = oracle.capacity(s, 1.1, 0.75, per_assignment=False)
    want["capacity.tokens"] = checksum(cap)
    cap[0] = 0
    pc = oracle.permute_capacity(s, r["topk_idx"], cap)
    Rc = int(pc["offsets"][-1])
    for k in ("kept", "offsets", "row_of"):
        want["cap." + k] = checksum(pc[k])
    want["cap.src_of"] = checksum(pc["src_of"][:Rc])
    b = oracle.balance(s, r["probs"], r["topk_idx"], 0.75)
    want["balance.f"], want["balance.P"], want["balance.loss"] = checksum(b["f"]), checksum(b["P"]), b["loss"]
    toks = np.array([36, 0, 17, 17, 5, 30], np.int32)
    e = oracle.experts(s, x, r["topk_idx"], r["topk_w"], w1, w3, w2, cv, W_c, tok_list=toks,
                       want_slots=True, want_h=True, want_alpha=True, row_of=pc["row_of"])
    for k in ("out", "slot_out", "h", "alpha1"):
        want["experts." + k] = checksum(e[k])
    ea = oracle.experts(s, x, r["topk_idx"], r["topk_w"], w1, w3, w2, cv, W_c)
    want["experts.out_all"] = checksum(ea["out"])
    gv = np.zeros((s.T, N))
    np.put_along_axis(gv, r["topk_idx"].astype(np.int64), r["topk_w"].astype(np.float64), axis=1)
    want["dense.out"] = checksum(oracle.dense(s, x, gv, w1, w3, w2, cv, W_c))
    with pytest.raises(ValueError):
        oracle.experts(s, x, r["topk_idx"], r["topk_w"], w1, w3, w2, cv, W_c,
                       tok_list=np.array([3, 37], np.int32))
    assert set(want) <= set(got)
    for k, v in want.items():
        assert abs(got[k] - v) <= 1e-12 * max(1.0, abs(v)), (k, got[k], v)


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2410_07348_amd import build as B
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib = str(tmp_path / "libmoepp_hostsan.so")
    host = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer"):
        host += ["-Xarch_host", f]
    flags = [f for f in B.FLAGS if f != "-O3"] + ["-O1", "-g"]
    run([hipcc] + flags + host + [os.path.join(B.CSRC, s) for s in B.SOURCES] + ["-o", lib])
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    exe = str(tmp_path / "boundary_san")
    run([clang, "-std=c11", "-g", "-O1", "-Wall", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
         "-I", os.path.join(ROOT, "include"), os.path.join(SAN, "boundary_main.c"), lib,
         "-Wl,-rpath," + str(tmp_path), "-o", exe])
    out = run([exe], env=ENV)
    assert out.strip().splitlines()[-1] == "ok", out
