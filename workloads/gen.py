"""Layer shapes and seeded tensor generation (no layer arithmetic here)."""
from __future__ import annotations

import dataclasses
import functools
from concurrent.futures import ThreadPoolExecutor

import numpy as np


@dataclasses.dataclass(frozen=True)
class LayerShape:
    """One MoE++ layer workload.

    Expert index order inside the N-way softmax: FFN experts first, then zero,
    copy and constant experts (the "zero/copy/constant" order of the paper's
    model table, Tab.2).
    """
    name: str
    T: int                 # tokens in the batch
    D: int                 # hidden size
    F: int                 # SwiGLU intermediate size
    n_ffn: int
    n_zero: int
    n_copy: int
    n_const: int
    k: int = 2             # top-k, 2 in every layer of the paper (Sec. 4.1)
    act: str = "bf16"      # activation / expert-weight type: "bf16" or "f32"
    residual: bool = True  # gating residual on (layer index j > 1, Eq.6)
    bias: str = "none"     # "none" | "normal" (N(0, 0.5) per expert) | "skew" | "tau<value>"
    seed: int = 20241007

    @property
    def N(self) -> int:
        return self.n_ffn + self.n_zero + self.n_copy + self.n_const

    @property
    def n_zc(self) -> int:
        return self.n_zero + self.n_copy + self.n_const

    def with_(self, **kw) -> "LayerShape":
        return dataclasses.replace(self, **kw)


# The benchmark configurations.  T is written as sequences x tokens.
WORKLOADS = {
    # fp32 end to end; the oracle finishes it in well under a second
    "tiny": LayerShape("tiny", T=256, D=128, F=256, n_ffn=4, n_zero=1, n_copy=1,
                       n_const=2, act="f32", seed=1001),
    "small": LayerShape("small", T=4 * 2048, D=1024, F=2048, n_ffn=8, n_zero=1,
                        n_copy=1, n_const=2, seed=1002),
    "mid": LayerShape("mid", T=8 * 2048, D=2048, F=1408, n_ffn=16, n_zero=1,
                      n_copy=1, n_const=2, bias="normal", seed=1003),
    "large": LayerShape("large", T=8 * 4096, D=4096, F=5632, n_ffn=16, n_zero=1,
                        n_copy=1, n_const=2, seed=1004),
    # vanilla MoE comparisons: same T/D/F/k, zero-computation experts disabled
    "large_vanilla20": LayerShape("large_vanilla20", T=8 * 4096, D=4096, F=5632,
                                  n_ffn=20, n_zero=0, n_copy=0, n_const=0,
                                  seed=1004),
    "large_vanilla16": LayerShape("large_vanilla16", T=8 * 4096, D=4096, F=5632,
                                  n_ffn=16, n_zero=0, n_copy=0, n_const=0,
                                  seed=1004),
    # about half of the top-2 slots on zero-computation experts, FFN expert 0
    # with four times the mean FFN load
    "skew": LayerShape("skew", T=8 * 2048, D=2048, F=1408, n_ffn=16, n_zero=1,
                       n_copy=1, n_const=2, bias="skew", seed=1005),
    "smallbatch": LayerShape("smallbatch", T=64, D=4096, F=5632, n_ffn=16,
                             n_zero=1, n_copy=1, n_const=2, seed=1006),
}

# Layer shapes of the paper's models (Tab.2): hidden 768 / intermediate 2048
# with 8, 16 or 32 FFN experts, hidden 1536 / intermediate 4096 with 16; zero /
# copy / constant experts 1/1/2 (1/1/6 with 32 FFN experts).  16 sequences of
# 2048 tokens (the paper's sequence length).  Used by bench.py --tau-sweep with
# bias = "tau<value>": the zero-computation experts get a common offset under
# which they take N_ZC / (tau N_FFN + N_ZC) of the assignments, the share the
# heterogeneous load-balance loss steers a trained model to (Sec. 3.3, Tab.1).
PAPER_MODELS = {
    "0.6B/(8+4)E": LayerShape("paper_0.6b", T=16 * 2048, D=768, F=2048, n_ffn=8, n_zero=1,
                              n_copy=1, n_const=2, seed=1010),
    "1B/(16+4)E": LayerShape("paper_1b", T=16 * 2048, D=768, F=2048, n_ffn=16, n_zero=1,
                             n_copy=1, n_const=2, seed=1011),
    "2B/(32+8)E": LayerShape("paper_2b", T=16 * 2048, D=768, F=2048, n_ffn=32, n_zero=1,
                             n_copy=1, n_const=6, seed=1012),
    "7B/(16+4)E": LayerShape("paper_7b", T=16 * 2048, D=1536, F=4096, n_ffn=16, n_zero=1,
                             n_copy=1, n_const=2, seed=1013),
}

# One Philox stream per tensor: key = (seed, TENSOR_IDS[name] [+ expert index]).
TENSOR_IDS = {"x": 1, "prev_gate": 2, "W_g": 3, "W_res": 4, "w1": 5, "w3": 6,
              "w2": 7, "const_vecs": 8, "W_c": 9, "bias": 10, "calib": 11}

WEIGHT_STD = 0.02   # "N(0, 0.02)" read as a standard deviation
BIAS_STD = 0.5


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round a float32 array to the nearest bfloat16 value (ties to even),
    in place, and return it (still float32-typed, low 16 bits zero)."""
    assert a.dtype == np.float32 and a.flags.c_contiguous
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    bits += np.uint32(0x7FFF) + lsb
    bits &= np.uint32(0xFFFF0000)
    return a


def _normal(seed: int, tid: int, sub: int, shape, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[seed, (tid << 32) | sub]))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def make_inputs(shape: LayerShape, threads: int = 8) -> dict:
    """All tensors of one layer call as float32 numpy arrays.

    With act == "bf16" the activation-typed tensors (x, w1, w3, w2,
    const_vecs) hold values that are exactly representable in bfloat16, so the
    oracle (which reads float32) and the GPU path (which reads bf16) consume
    the same numbers.  Router-side tensors are float32 in every workload.

    Logical layouts: x [T,D]; prev_gate [T,N]; W_g [N,D]; W_res [N,N];
    w1, w3 [n_ffn,F,D]; w2 [n_ffn,D,F]; const_vecs [n_const,D];
    W_c [n_const,2,D]; bias [N] or None.
    """
    s = shape
    bf = s.act == "bf16"
    sd = s.seed

    def act_tensor(name, sub, shp, std):
        a = _normal(sd, TENSOR_IDS[name], sub, shp, std)
        return round_to_bf16(a) if bf else a

    out = {}
    out["x"] = act_tensor("x", 0, (s.T, s.D), 1.0)
    if s.residual:
        out["prev_gate"] = _normal(sd, TENSOR_IDS["prev_gate"], 0, (s.T, s.N), 1.0)
        out["W_res"] = _normal(sd, TENSOR_IDS["W_res"], 0, (s.N, s.N), WEIGHT_STD)
    else:
        out["prev_gate"] = None
        out["W_res"] = None
    out["W_g"] = _normal(sd, TENSOR_IDS["W_g"], 0, (s.N, s.D), WEIGHT_STD)
    out["const_vecs"] = act_tensor("const_vecs", 0, (s.n_const, s.D), WEIGHT_STD)
    out["W_c"] = _normal(sd, TENSOR_IDS["W_c"], 0, (s.n_const, 2, s.D), WEIGHT_STD)

    for name, shp in (("w1", (s.F, s.D)), ("w3", (s.F, s.D)), ("w2", (s.D, s.F))):
        full = np.empty((s.n_ffn,) + shp, dtype=np.float32)

        def fill(e, name=name, shp=shp, full=full):
            full[e] = act_tensor(name, e, shp, WEIGHT_STD)

        if s.n_ffn * shp[0] * shp[1] > (1 << 24) and threads > 1:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(fill, range(s.n_ffn)))
        else:
            for e in range(s.n_ffn):
                fill(e)
        out[name] = full
    out["bias"] = make_router_bias(s)
    return out


def make_router_bias(shape: LayerShape):
    """Additive per-expert router bias (a benchmark knob, not in the paper)."""
    s = shape
    if s.bias == "none":
        return None
    if s.bias == "normal":
        return _normal(s.seed, TENSOR_IDS["bias"], 0, (s.N,), BIAS_STD)
    if s.bias == "skew":
        b_zc, b_hot = skew_bias_gaussian_model(s.D, s.n_ffn, s.n_zc, s.k,
                                               s.residual, s.seed)
        b = np.zeros(s.N, dtype=np.float32)
        b[s.n_ffn:] = b_zc
        b[0] = b_hot
        return b
    if s.bias.startswith("tau"):
        tau = float(s.bias[3:])
        share = s.n_zc / (tau * s.n_ffn + s.n_zc)
        b_zc, _ = skew_bias_gaussian_model(s.D, s.n_ffn, s.n_zc, s.k, s.residual, s.seed,
                                           zc_share=share, hot_ratio=1.0)
        b = np.zeros(s.N, dtype=np.float32)
        b[s.n_ffn:] = b_zc
        return b
    raise ValueError(s.bias)


@functools.lru_cache(maxsize=None)
def skew_bias_gaussian_model(D: int, n_ffn: int, n_zc: int, k: int,
                             residual: bool, seed: int,
                             zc_share: float = 0.5, hot_ratio: float = 4.0):
    """Find (b_zc, b_hot) for the skewed-routing workload.

    The layer's logits for random inputs are close to i.i.d. Gaussians with
    variance D*WEIGHT_STD^2 (+ N*WEIGHT_STD^2 from the gating residual); this
    draws such stand-in logits (seeded) and bisects the two offsets until the
    k largest of b + logits land on zero-computation experts for `zc_share`
    of the slots and on FFN expert 0 `hot_ratio` times as often as on the
    other FFN experts on average.  Only Gaussian stand-ins are used, so the
    result does not depend on any layer code.
    """
    N = n_ffn + n_zc
    var = D * WEIGHT_STD ** 2 + (N * WEIGHT_STD ** 2 if residual else 0.0)
    z = _normal(seed, TENSOR_IDS["calib"], 0, (1 << 15, N), float(np.sqrt(var)))

    def shares(b_zc, b_hot):
        l = z.copy()
        l[:, n_ffn:] += b_zc
        l[:, 0] += b_hot
        top = np.argpartition(-l, k - 1, axis=1)[:, :k]
        cnt = np.bincount(top.ravel(), minlength=N).astype(np.float64)
        zc = cnt[n_ffn:].sum() / cnt.sum()
        hot = cnt[0] / max(cnt[1:n_ffn].mean(), 1.0)
        return zc, hot

    b_zc, b_hot = 0.0, 0.0
    for _ in range(4):                       # alternate the two bisections
        lo, hi = -4.0, 8.0
        for _ in range(16):
            mid = 0.5 * (lo + hi)
            if shares(mid, b_hot)[0] < zc_share:
                lo = mid
            else:
                hi = mid
        b_zc = 0.5 * (lo + hi)
        lo, hi = -4.0, 8.0
        for _ in range(16):
            mid = 0.5 * (lo + hi)
            if shares(b_zc, mid)[1] < hot_ratio:
                lo = mid
            else:
                hi = mid
        b_hot = 0.5 * (lo + hi)
    return float(np.float32(b_zc)), float(np.float32(b_hot))


def ffn_work_fraction(tau: float, n_ffn: int, n_zc: int) -> float:
    """FFN work of an MoE++ layer relative to a vanilla MoE with the same FFN
    experts, as the paper's complexity table states it (Tab.1, Sec. 3.4)."""
    return tau * n_ffn / (tau * n_ffn + n_zc)


def n_const_rule(n_ffn: int, n_zero: int = 1, n_copy: int = 1) -> int:
    """Number of constant experts the paper recommends (Eq.10)."""
    return max(n_ffn // 4 - n_zero - n_copy, 1)
