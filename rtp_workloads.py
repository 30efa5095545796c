"""Seeded synthetic inputs for the rotated-shard linear layer.

This module is the only thing the CPU oracle's tests and the HIP path's tests
and benchmark share.  It draws numbers and rounds them to the storage type;
it holds none of the method's arithmetic (no products, no schedule).

Recipe: numpy `default_rng(seed)`, fp32 draws, in the order X, the weights in
the order the workload lists them, dY (then any extra input).  For a bf16
workload every array is rounded to bf16 (round to nearest even) and kept as
fp32 holding exactly those values, so that the fp64 oracle and the GPU see the
same numbers.
"""
from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str            # "linear" | "linear_in" | "mlp_gelu" | "swiglu" | "linears"
    T: int               # local tokens of the one worker
    I: int               # in-features
    O: int               # out-features of the (first) partitioned matrix
    n: int               # partition factor N (virtual shards)
    dtype: str           # "f32" | "bf16" | "f16"
    mode: str            # "double_buffer" | "inplace_staged"
    O2: int = 0          # out-features of the second (input-partitioned) matrix
    w_dist: tuple = ("normal", 0.02)
    extra: dict = field(default_factory=dict)

    @property
    def flops(self):
        """fwd+bwd flops, 6 T I O per matrix; elementwise work not counted."""
        if self.kind in ("linear", "linear_in"):
            return 6 * self.T * self.I * self.O
        if self.kind == "mlp_gelu":
            return 6 * self.T * (self.I * self.O + self.O * self.O2)
        if self.kind == "swiglu":
            return 6 * self.T * (2 * self.I * self.O + self.O * self.O2)
        if self.kind == "moe_swiglu":      # every token goes through one expert
            return 6 * self.T * (2 * self.I * self.O + self.O * self.O2)
        if self.kind == "linears":
            return sum(6 * self.T * i * o for (_, o, i) in self.extra["matrices"])
        raise ValueError(self.kind)


# The five configurations of the benchmark definition, at their full sizes.
CONFIGS = {
    "cfg1_linear_f32": Workload("cfg1_linear_f32", "linear", T=64, I=256, O=512, n=4, dtype="f32",
                                mode="double_buffer", w_dist=("uniform", 1.0 / 16.0)),
    "cfg2_gpt2s_mlp": Workload("cfg2_gpt2s_mlp", "mlp_gelu", T=8192, I=768, O=3072, O2=768, n=8,
                               dtype="bf16", mode="double_buffer"),
    "cfg3_d2048_proj": Workload("cfg3_d2048_proj", "linears", T=8192, I=2048, O=6144, n=8, dtype="bf16",
                                mode="double_buffer",
                                extra={"matrices": (("qkv", 6144, 2048), ("out", 2048, 2048),
                                                    ("up", 8192, 2048), ("down", 2048, 8192))}),
    "cfg4_llama7b_swiglu": Workload("cfg4_llama7b_swiglu", "swiglu", T=4096, I=4096, O=11008, O2=4096,
                                    n=8, dtype="bf16", mode="inplace_staged"),
    "cfg5_large_mlp": Workload("cfg5_large_mlp", "mlp_gelu", T=2048, I=8192, O=28672, O2=8192, n=16,
                               dtype="bf16", mode="inplace_staged", w_dist=("normal", 0.01)),
}


# Expert partition (the paper names the layer but gives no sizes): eight experts of the shape of a
# widely used open mixture-of-experts model's feed-forward block, one expert per token, 8192 local
# tokens, load skewed as (e + 1)^-1.  `make_moe_inputs` draws it.
MOE_CONFIGS = {
    "moe_8x_swiglu": Workload("moe_8x_swiglu", "moe_swiglu", T=8192, I=4096, O=14336, O2=4096, n=8, dtype="bf16",
                              mode="inplace_staged", extra={"skew": 1.0}),
}


def round_to_bf16(x):
    """fp32 array -> fp32 array holding the nearest bf16 values (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # finite inputs only: the carry of the rounding add never reaches the sign bit
    r = (u >> np.uint32(16)) & np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r &= np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(x.shape)


def _store(x, dtype):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)   # nearest fp16 value, ties to even
    return round_to_bf16(x) if dtype == "bf16" else x


def _weight(rng, shape, dist):
    kind, scale = dist
    if kind == "normal":
        return (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)).astype(np.float32)
    if kind == "uniform":
        return rng.uniform(-scale, scale, size=shape).astype(np.float32)
    raise ValueError(kind)


def make_inputs(wl: Workload, seed: int = 0, grad0: bool = False):
    """Returns a dict of fp32 arrays (bf16-exact for bf16 workloads).

    With grad0=True also draws the content the travelling gradient shards
    hold on arrival (`G0_*`), so that accumulate-versus-overwrite mistakes
    show; otherwise gradients start from zero."""
    rng = np.random.default_rng(seed)
    d = wl.dtype
    out = {}
    if wl.kind in ("linear", "linear_in"):
        out["X"] = _store(rng.standard_normal((wl.T, wl.I), dtype=np.float32), d)
        out["W"] = _store(_weight(rng, (wl.O, wl.I), wl.w_dist), d)
        out["dY"] = _store(rng.standard_normal((wl.T, wl.O), dtype=np.float32), d)
        names = [("W", (wl.O, wl.I))]
    elif wl.kind == "mlp_gelu":
        out["X"] = _store(rng.standard_normal((wl.T, wl.I), dtype=np.float32), d)
        out["W1"] = _store(_weight(rng, (wl.O, wl.I), wl.w_dist), d)
        out["W2"] = _store(_weight(rng, (wl.O2, wl.O), wl.w_dist), d)
        out["dY"] = _store(rng.standard_normal((wl.T, wl.O2), dtype=np.float32), d)
        names = [("W1", (wl.O, wl.I)), ("W2", (wl.O2, wl.O))]
    elif wl.kind == "swiglu":
        out["X"] = _store(rng.standard_normal((wl.T, wl.I), dtype=np.float32), d)
        out["Wg"] = _store(_weight(rng, (wl.O, wl.I), wl.w_dist), d)
        out["Wu"] = _store(_weight(rng, (wl.O, wl.I), wl.w_dist), d)
        out["Wd"] = _store(_weight(rng, (wl.O2, wl.O), wl.w_dist), d)
        out["dY"] = _store(rng.standard_normal((wl.T, wl.O2), dtype=np.float32), d)
        names = [("Wg", (wl.O, wl.I)), ("Wu", (wl.O, wl.I)), ("Wd", (wl.O2, wl.O))]
    elif wl.kind == "linears":
        mats = wl.extra["matrices"]
        widths = sorted({i for (_, _, i) in mats}, key=lambda w: [i for (_, _, i) in mats].index(w))
        for w in widths:
            out[f"X_{w}"] = _store(rng.standard_normal((wl.T, w), dtype=np.float32), d)
        names = []
        for (nm, o, i) in mats:
            out[f"W_{nm}"] = _store(_weight(rng, (o, i), wl.w_dist), d)
            names.append((f"W_{nm}", (o, i)))
        for (nm, o, i) in mats:
            out[f"dY_{nm}"] = _store(rng.standard_normal((wl.T, o), dtype=np.float32), d)
    else:
        raise ValueError(wl.kind)
    if grad0:
        for nm, shape in names:
            # gradient shards are kept in fp32 on the GPU, so no bf16 rounding here
            out["G0_" + nm] = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.5)
    return out


def make_integer_inputs(wl: Workload, seed: int = 0, lo: int = -2, hi: int = 2):
    """Same shapes, entries uniform in {lo..hi}: exact in bf16, and every
    partial sum of a contraction stays an integer below 2^24, so any order of
    summation in fp32 gives the same bits."""
    rng = np.random.default_rng(seed)
    assert wl.kind in ("linear", "linear_in")
    assert max(abs(lo), abs(hi)) ** 2 * max(wl.T, wl.I, wl.O) < 2 ** 24
    out = {
        "X": rng.integers(lo, hi + 1, size=(wl.T, wl.I)).astype(np.float32),
        "W": rng.integers(lo, hi + 1, size=(wl.O, wl.I)).astype(np.float32),
        "dY": rng.integers(lo, hi + 1, size=(wl.T, wl.O)).astype(np.float32),
    }
    return out


def make_moe_inputs(T, I, O, O2, n, dtype="bf16", gated=False, seed=0, skew=1.0, w_scale=0.05, grad0=True):
    """Inputs of an expert-partitioned layer: n experts of one shape, and one expert id per token.

    The paper defines no router, so the routing is a drawn input: token t goes to expert e with
    probability proportional to (e + 1)^-skew (skew 0: uniform load; 1: the few-busy-many-idle
    load mixture-of-experts layers show), independently per token.  Draw order: X, the experts in
    order (each matrix in order), dY, route, then the arriving gradients."""
    rng = np.random.default_rng(seed)
    shapes = [(O, I), (O, I), (O2, O)] if gated else [(O, I), (O2, O)]
    out = {"X": _store(rng.standard_normal((T, I), dtype=np.float32), dtype)}
    out["experts"] = [tuple(_store(_weight(rng, sh, ("normal", w_scale)), dtype) for sh in shapes) for _ in range(n)]
    out["dY"] = _store(rng.standard_normal((T, O2), dtype=np.float32), dtype)
    p = (np.arange(n) + 1.0) ** -float(skew)
    out["route"] = rng.choice(n, size=T, p=p / p.sum()).astype(np.int32)
    if grad0:
        out["G0"] = [tuple(rng.standard_normal(sh, dtype=np.float32) * np.float32(0.5) for sh in shapes)
                     for _ in range(n)]
    return out


def scaled(wl: Workload, name: str, **kw) -> Workload:
    """A smaller or reshaped copy of a workload for parity tests."""
    from dataclasses import replace
    return replace(wl, name=name, **kw)
