"""ctypes binding of libmoepp.so; same names as include/moepp.h."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int32, c_size_t, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
F32, BF16 = 0, 1
OK, EINVAL, EUNSUPPORTED, ENOMEM, EHIP = 0, -1, -2, -3, -4
KERNEL_NAMES = ("router", "perm_hist", "perm_scan", "perm_scatter", "gemm1", "gemm2",
                "combine", "balance")

# every symbol include/moepp.h declares
EXPORTS = ("moepp_workspace_bytes", "moepp_packed_bytes", "moepp_create", "moepp_destroy",
           "moepp_pack_experts", "moepp_set_router_bias", "moepp_layer_forward",
           "moepp_route", "moepp_permute", "moepp_expert_ffn", "moepp_combine",
           "moepp_get_routing", "moepp_get_intermediates", "moepp_set_timing",
           "moepp_get_timing", "moepp_set_variant", "moepp_mfma_ceiling", "moepp_status_str",
           "moepp_capacity", "moepp_set_capacity", "moepp_get_kept", "moepp_set_balance",
           "moepp_get_balance", "moepp_layer_forward_static", "moepp_stream_ceiling")


class MoeppError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (%d)" % (what, status_str(status), status))


class Desc(ctypes.Structure):
    """moepp_desc"""
    _fields_ = [(n, c_int32) for n in ("T_max", "D", "F", "n_ffn", "n_zero", "n_copy",
                                       "n_const", "k", "act")]

    @property
    def N(self):
        return self.n_ffn + self.n_zero + self.n_copy + self.n_const


class _Experts(ctypes.Structure):
    _fields_ = [("w1", c_void_p), ("w3", c_void_p), ("w2", c_void_p)]


def lib_path() -> str:
    return os.path.join(HERE, "libmoepp.so")


_lib = None


def load_library(build_if_missing: bool = True):
    """Load libmoepp.so.  Builds it with hipcc only when no built library is
    present; raises if it cannot be loaded (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        if not build_if_missing:
            raise FileNotFoundError(path)
        from . import build as _build
        _build.build()
    L = ctypes.CDLL(path)
    vp, i32, f32p = c_void_p, c_int32, c_void_p
    L.moepp_workspace_bytes.restype = c_size_t
    L.moepp_workspace_bytes.argtypes = [POINTER(Desc)]
    L.moepp_packed_bytes.restype = c_size_t
    L.moepp_packed_bytes.argtypes = [POINTER(Desc)]
    L.moepp_create.argtypes = [POINTER(Desc), vp, c_size_t, POINTER(vp)]
    L.moepp_destroy.argtypes = [vp]
    L.moepp_pack_experts.argtypes = [vp, vp, POINTER(_Experts), vp, c_size_t]
    L.moepp_set_router_bias.argtypes = [vp, f32p]
    L.moepp_layer_forward.argtypes = [vp, vp, i32, vp, f32p, f32p, f32p, vp, vp, f32p, i32,
                                      vp, f32p]
    L.moepp_layer_forward_static.argtypes = [POINTER(Desc), vp, i32, vp, f32p, f32p, f32p, vp, vp,
                                             f32p, i32, vp, f32p]
    L.moepp_route.argtypes = [vp, vp, i32, vp, f32p, f32p, f32p, f32p, i32, f32p]
    L.moepp_permute.argtypes = [vp, vp, i32, i32]
    L.moepp_expert_ffn.argtypes = [vp, vp, i32, vp, vp, i32]
    L.moepp_combine.argtypes = [vp, vp, i32, vp, vp, i32, vp]
    L.moepp_get_routing.argtypes = [vp] + [POINTER(vp)] * 6
    L.moepp_get_intermediates.argtypes = [vp] + [POINTER(vp)] * 3
    L.moepp_set_timing.argtypes = [vp, i32]
    L.moepp_get_timing.argtypes = [vp, POINTER(c_float)]
    L.moepp_set_variant.argtypes = [vp, i32]
    L.moepp_mfma_ceiling.argtypes = [vp, vp, c_size_t, i32, POINTER(ctypes.c_double)]
    L.moepp_stream_ceiling.argtypes = [vp, vp, c_size_t, i32, POINTER(ctypes.c_double)]
    L.moepp_capacity.argtypes = [POINTER(Desc), i32, i32, ctypes.c_double, ctypes.c_double,
                                 i32, POINTER(c_int32)]
    L.moepp_set_capacity.argtypes = [vp, POINTER(c_int32)]
    L.moepp_get_kept.argtypes = [vp, POINTER(vp)]
    L.moepp_set_balance.argtypes = [vp, ctypes.c_double]
    L.moepp_get_balance.argtypes = [vp] + [POINTER(vp)] * 3
    L.moepp_status_str.restype = c_char_p
    L.moepp_status_str.argtypes = [i32]
    for n in EXPORTS:
        if n not in ("moepp_workspace_bytes", "moepp_packed_bytes", "moepp_status_str"):
            getattr(L, n).restype = c_int32
    _lib = L
    return L


def status_str(status: int) -> str:
    return load_library().moepp_status_str(status).decode()


def _check(status, what):
    if status != OK:
        raise MoeppError(status, what)


def _ptr(t, dtype=None, device=None):
    """Device address of a torch tensor (None -> NULL).  The library reads raw
    memory: a tensor of another type, on another device or not contiguous would
    be misread without any error, so those are refused here."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected a %s tensor, got %s" % (dtype, t.dtype))
    if device is not None and t.device != device:
        raise ValueError("tensor is on %s, the layer on %s" % (t.device, device))
    return c_void_p(t.data_ptr())


def mfma_ceiling(iters=20000, reps=3, device="cuda:0"):
    """Sustained bf16 MFMA rate (TFLOP/s) on pseudo-random operands, timed with
    events on the current stream; the best of `reps` launches."""
    import torch
    L = load_library()
    dev = torch.device(device)
    scratch = torch.empty(512 * 1024, dtype=torch.uint8, device=dev)
    flops = ctypes.c_double()
    best = 0.0
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        stream = torch.cuda.current_stream(dev)
        e0.record(stream)
        _check(L.moepp_mfma_ceiling(c_void_p(stream.cuda_stream), _ptr(scratch), scratch.numel(),
                                    iters, byref(flops)), "moepp_mfma_ceiling")
        e1.record(stream)
        e1.synchronize()
        best = max(best, flops.value / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best


def stream_ceiling(mode=0, nbytes=1 << 30, reps=3, device="cuda:0"):
    """GB/s of a kernel that only reads (mode 0) or copies (mode 1) `nbytes`, timed with
    events on the current stream; the best of `reps` launches after one warm-up."""
    import torch
    L = load_library()
    dev = torch.device(device)
    buf = torch.ones(nbytes, dtype=torch.uint8, device=dev)
    moved = ctypes.c_double()
    stream = torch.cuda.current_stream(dev)
    best = 0.0
    for rep in range(reps + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        _check(L.moepp_stream_ceiling(c_void_p(stream.cuda_stream), _ptr(buf), nbytes, mode,
                                      byref(moved)), "moepp_stream_ceiling")
        e1.record(stream)
        e1.synchronize()
        if rep:
            best = max(best, moved.value / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return best


STATIC_SCRATCH_BYTES = 32 << 20      # MOEPP_STATIC_SCRATCH_BYTES


def layer_forward_static(desc, x, prev_gate, W_g, W_res, experts, const_vecs, W_c, k, out,
                         out_gate, stream=None):
    """moepp_layer_forward_static: the forward pass on the library's own static
    scratch.  Every tensor, `out` and `out_gate` included, is the caller's; this
    function allocates nothing."""
    import torch
    L = load_library()
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    act = torch.bfloat16 if desc.act == BF16 else torch.float32
    dev = x.device
    _check(L.moepp_layer_forward_static(
        byref(desc), c_void_p(stream), x.shape[0], _ptr(x, act, dev),
        _ptr(prev_gate, torch.float32, dev), _ptr(W_g, torch.float32, dev),
        _ptr(W_res, torch.float32, dev), _ptr(experts, torch.uint8, dev),
        _ptr(const_vecs, act, dev), _ptr(W_c, torch.float32, dev), k, _ptr(out, act, dev),
        _ptr(out_gate, torch.float32, dev)), "moepp_layer_forward_static")


class Layer:
    """One MoE++ layer context.  Tensors are torch CUDA tensors; `act` is
    "bf16" or "f32".  Methods mirror the C entry points one to one."""

    def __init__(self, T_max, D, F, n_ffn, n_zero, n_copy, n_const, k=2, act="bf16",
                 device="cuda:0"):
        import torch
        self.torch = torch
        self.L = load_library()
        self.desc = Desc(T_max, D, F, n_ffn, n_zero, n_copy, n_const, k,
                         BF16 if act == "bf16" else F32)
        self.act_dtype = torch.bfloat16 if act == "bf16" else torch.float32
        self.device = torch.device(device)
        nbytes = self.L.moepp_workspace_bytes(byref(self.desc))
        if nbytes == 0:
            probe = c_void_p()
            st = self.L.moepp_create(byref(self.desc), c_void_p(256), 0, byref(probe))
            raise MoeppError(st, "moepp_create")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.ctx = c_void_p()
        _check(self.L.moepp_create(byref(self.desc), _ptr(self.workspace), nbytes,
                                   byref(self.ctx)), "moepp_create")
        self._bias = None
        self.last_T = 0
        self.last_k = k

    def close(self):
        if getattr(self, "ctx", None):
            self.L.moepp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers -----------------------------------------------------------
    def _act(self, t):
        return _ptr(t, self.act_dtype, self.device)

    def _f32(self, t):
        return _ptr(t, self.torch.float32, self.device)

    def _stream(self):
        return c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def _view(self, ptr, n, dtype):
        off = ptr - self.workspace.data_ptr()
        nb = n * self.torch.empty(0, dtype=dtype).element_size()
        assert 0 <= off and off + nb <= self.workspace.numel()
        return self.workspace[off:off + nb].view(dtype)

    # -- C entry points ----------------------------------------------------
    def pack_experts(self, w1, w3, w2):
        t = self.torch
        nbytes = self.L.moepp_packed_bytes(byref(self.desc))
        packed = t.empty(nbytes, dtype=t.uint8, device=self.device)
        for w in (w1, w3, w2):
            self._act(w)
        ex = _Experts(w1.data_ptr() if w1 is not None else None,
                      w3.data_ptr() if w3 is not None else None,
                      w2.data_ptr() if w2 is not None else None)
        _check(self.L.moepp_pack_experts(self.ctx, self._stream(), byref(ex), _ptr(packed),
                                         nbytes), "moepp_pack_experts")
        return packed

    def set_router_bias(self, bias):
        self._bias = bias          # keep the tensor alive: the library keeps the pointer
        _check(self.L.moepp_set_router_bias(self.ctx, self._f32(bias)), "moepp_set_router_bias")

    def set_variant(self, v):
        _check(self.L.moepp_set_variant(self.ctx, v), "moepp_set_variant")

    def set_timing(self, on):
        _check(self.L.moepp_set_timing(self.ctx, 1 if on else 0), "moepp_set_timing")

    def get_timing(self):
        ms = (c_float * len(KERNEL_NAMES))()
        _check(self.L.moepp_get_timing(self.ctx, ms), "moepp_get_timing")
        return dict(zip(KERNEL_NAMES, [float(v) for v in ms]))

    def layer_forward(self, x, prev_gate, W_g, W_res, experts, const_vecs, W_c, k=None,
                      out=None, out_gate=None):
        t = self.torch
        k = self.desc.k if k is None else k
        T = x.shape[0]
        if out is None:
            out = t.empty((T, self.desc.D), dtype=self.act_dtype, device=self.device)
        if out_gate is None:
            out_gate = t.empty((T, self.desc.N), dtype=t.float32, device=self.device)
        _check(self.L.moepp_layer_forward(self.ctx, self._stream(), T, self._act(x),
                                          self._f32(prev_gate), self._f32(W_g), self._f32(W_res),
                                          _ptr(experts, t.uint8, self.device),
                                          self._act(const_vecs), self._f32(W_c), k,
                                          self._act(out), self._f32(out_gate)),
               "moepp_layer_forward")
        self.last_T, self.last_k = T, k
        return out, out_gate

    def route(self, x, prev_gate, W_g, W_res, W_c, k=None, out_gate=None):
        t = self.torch
        k = self.desc.k if k is None else k
        T = x.shape[0]
        if out_gate is None:
            out_gate = t.empty((T, self.desc.N), dtype=t.float32, device=self.device)
        _check(self.L.moepp_route(self.ctx, self._stream(), T, self._act(x),
                                  self._f32(prev_gate), self._f32(W_g), self._f32(W_res),
                                  self._f32(W_c), k, self._f32(out_gate)), "moepp_route")
        self.last_T, self.last_k = T, k
        return out_gate

    def permute(self, T=None, k=None):
        T = self.last_T if T is None else T
        k = self.last_k if k is None else k
        _check(self.L.moepp_permute(self.ctx, self._stream(), T, k), "moepp_permute")
        self.last_T, self.last_k = T, k

    def expert_ffn(self, x, experts, k=None):
        k = self.last_k if k is None else k
        _check(self.L.moepp_expert_ffn(self.ctx, self._stream(), x.shape[0], self._act(x),
                                       _ptr(experts, self.torch.uint8, self.device), k),
               "moepp_expert_ffn")

    def combine(self, x, const_vecs, k=None, out=None):
        t = self.torch
        k = self.last_k if k is None else k
        if out is None:
            out = t.empty((x.shape[0], self.desc.D), dtype=self.act_dtype, device=self.device)
        _check(self.L.moepp_combine(self.ctx, self._stream(), x.shape[0], self._act(x),
                                    self._act(const_vecs), k, self._act(out)), "moepp_combine")
        return out

    def get_routing(self):
        """Views into the workspace: topk_idx/topk_w [T,k], counts [N],
        offsets [n_ffn+1], row_of/src_of [T*k]."""
        t = self.torch
        p = [c_void_p() for _ in range(6)]
        _check(self.L.moepp_get_routing(self.ctx, *[byref(q) for q in p]), "moepp_get_routing")
        T, k, d = self.last_T, self.last_k, self.desc
        return {
            "topk_idx": self._view(p[0].value, T * k, t.int32).view(T, k),
            "topk_w": self._view(p[1].value, T * k, t.float32).view(T, k),
            "counts": self._view(p[2].value, d.N, t.int32),
            "offsets": self._view(p[3].value, d.n_ffn + 1, t.int32),
            "row_of": self._view(p[4].value, T * k, t.int32),
            "src_of": self._view(p[5].value, T * k, t.int32),
        }

    def capacity(self, T, gamma, tau, k=None, per_assignment=True):
        """Expert capacities C_i of Eq.8 for a call with T tokens: list of N ints
        (per_assignment=False: Eq.8 with T tokens literally instead of T*k assignments)."""
        cap = (c_int32 * self.desc.N)()
        _check(self.L.moepp_capacity(byref(self.desc), T, self.desc.k if k is None else k,
                                     gamma, tau, 1 if per_assignment else 0, cap), "moepp_capacity")
        return [int(v) for v in cap]

    def set_capacity(self, cap):
        """Per-expert capacities for the following calls (None: unlimited)."""
        if cap is None:
            _check(self.L.moepp_set_capacity(self.ctx, None), "moepp_set_capacity")
            return
        arr = (c_int32 * self.desc.N)(*[int(v) for v in cap])
        _check(self.L.moepp_set_capacity(self.ctx, arr), "moepp_set_capacity")

    def get_kept(self):
        p = c_void_p()
        _check(self.L.moepp_get_kept(self.ctx, byref(p)), "moepp_get_kept")
        return self._view(p.value, self.desc.N, self.torch.int32)

    def set_balance(self, tau):
        """Collect f_i, P_i, L_b of Eq.7 with this tau (<= 0: off)."""
        _check(self.L.moepp_set_balance(self.ctx, float(tau)), "moepp_set_balance")

    def get_balance(self):
        p = [c_void_p() for _ in range(3)]
        _check(self.L.moepp_get_balance(self.ctx, *[byref(q) for q in p]), "moepp_get_balance")
        f32, N = self.torch.float32, self.desc.N
        return {"f": self._view(p[0].value, N, f32), "P": self._view(p[1].value, N, f32),
                "loss": self._view(p[2].value, 1, f32)}

    def get_intermediates(self, R=None):
        """alpha1 [T,n_const]; h [R,F]; yffn [R,D] (R rows reach an FFN)."""
        t = self.torch
        p = [c_void_p() for _ in range(3)]
        _check(self.L.moepp_get_intermediates(self.ctx, *[byref(q) for q in p]),
               "moepp_get_intermediates")
        T, d = self.last_T, self.desc
        if R is None:
            R = int(self.get_routing()["offsets"][-1].item()) if d.n_ffn else 0
        out = {"alpha1": self._view(p[0].value, T * d.n_const, t.float32).view(T, d.n_const)}
        if d.n_ffn:
            # h is stored in slabs of 32 columns over T_max*k rows: gather it to [R,F]
            slots, cols = d.T_max * d.k, []
            raw = self._view(p[1].value, slots * d.F, self.act_dtype)
            for s0 in range(0, d.F, 32):
                w = min(32, d.F - s0)
                cols.append(raw[s0 * slots: s0 * slots + slots * w].view(slots, w)[:R])
            out["h"] = t.cat(cols, dim=1)
            out["yffn"] = self._view(p[2].value, R * d.D, self.act_dtype).view(R, d.D)
        return out
