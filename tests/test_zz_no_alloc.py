"""moepp_layer_forward_static (the entry point that allocates nothing: its
scratch is a static array in the library's device code) against
moepp_layer_forward on a caller-provided workspace, through the C ABI: the
same kernels on the same inputs, so every output must be bit-identical.  Two
calls in a row, the second with fewer tokens (it must not be disturbed by what
the first left in the shared array), then a third, larger one with another
shape.  Needs a real MI355X: run with -m gpu."""
import ctypes

import numpy as np
import pytest

import paper_2410_07348_amd as M
from workloads import LayerShape, make_inputs

from helpers import check_layer, gpu_forward, make_layer, to_device

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def run_both(s, T_max):
    import torch
    inp = make_inputs(s)
    dev = to_device(s, inp)
    L = make_layer(s, T_max=T_max)
    assert L.workspace.numel() <= M.STATIC_SCRATCH_BYTES
    packed = L.pack_experts(dev["w1"], dev["w3"], dev["w2"])
    ref_out, ref_gate = L.layer_forward(dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], packed,
                                        dev["const_vecs"], dev["W_c"], k=s.k)
    torch.cuda.synchronize()
    out = torch.full_like(ref_out, float("nan"))
    gate = torch.full_like(ref_gate, float("nan"))
    free0 = torch.cuda.mem_get_info()[0]
    M.layer_forward_static(L.desc, dev["x"], dev["prev_gate"], dev["W_g"], dev["W_res"], packed,
                           dev["const_vecs"], dev["W_c"], s.k, out, gate)
    torch.cuda.synchronize()
    say("free device memory before / after the call:", free0, torch.cuda.mem_get_info()[0])
    assert torch.equal(out, ref_out), "out differs"
    assert torch.equal(gate, ref_gate), "out_gate differs"
    return inp, out, gate


def test_static_scratch_forward_equals_the_workspace_forward_on_two_calls_in_a_row():
    big = LayerShape("static_a", T=700, D=512, F=768, n_ffn=6, n_zero=1, n_copy=1, n_const=2, k=2,
                     act="bf16", seed=3101)
    say("static scratch: first call", big)
    run_both(big, T_max=700)
    small = big.with_(name="static_b", T=93, seed=3102)
    say("static scratch: second, smaller call", small)
    inp, out, gate = run_both(small, T_max=700)
    # and right against the oracle, not only equal to the other entry point
    res = gpu_forward(small, inp, intermediates=False)
    assert np.array_equal(res["out"], out.float().cpu().numpy().astype(np.float64))
    say("errs", check_layer(small, inp, res, check_inter=False))
    other = LayerShape("static_c", T=1500, D=256, F=256, n_ffn=9, n_zero=2, n_copy=1, n_const=1, k=3,
                       act="f32", seed=3103)
    say("static scratch: third call, another shape and type", other)
    run_both(other, T_max=1500)


def test_static_scratch_forward_rejects_what_does_not_fit():
    import torch
    L = M.load_library()
    d = M.Desc(1 << 16, 4096, 5632, 16, 1, 1, 2, 2, M.BF16)
    assert L.moepp_workspace_bytes(ctypes.byref(d)) > M.STATIC_SCRATCH_BYTES
    x = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    p = ctypes.c_void_p(x.data_ptr())
    st = L.moepp_layer_forward_static(ctypes.byref(d), None, 16, p, None, p, None, p, p, p, 2, p, p)
    assert st == -3 and L.moepp_status_str(st) == b"buffer too small"
    # T = 0 is a no-op that reads no pointer
    d2 = M.Desc(64, 256, 256, 4, 1, 1, 2, 2, M.BF16)
    assert L.moepp_layer_forward_static(ctypes.byref(d2), None, 0, None, None, None, None, None, None,
                                        None, 2, None, None) == 0
