"""Benchmark of the rotated-shard MLP unit on one MI355X.

A "step" is one whole pass of the hot path over one batch: the forward
rotation (N steps) and the backward rotation (N steps) of the Llama-7B-shaped
SwiGLU MLP unit with N = 8 virtual shards staged in place on a second stream.
Inputs are synthetic, seeded and resident in HBM before the timed region.

Prints ONE JSON line: whole-job TFLOP/s (6 T I O flops per matrix), the
roofline of the dominant kernel (per-launch HIP-event timing in an
instrumented repeat of the same steps), the fraction of shard staging hidden
under compute (three-run method), and the CPU oracle timed on a bounded
token sample on this host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published)
PEAK_F32_VECTOR_TFLOPS = 157.3   # fp32 vector ALU peak (the fp32 correctness path runs plain FMA kernels)
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg4_llama7b_swiglu")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true", help="skip the three-run staging-overlap measurement")
    ap.add_argument("--schedule", default="default", choices=["default", "pipelined", "grouped", "stepwise", "fused"],
                    help="launch schedule of the MLP unit: default (forward: independent GEMMs of a step in one launch; "
                         "backward: one launch per GEMM, weight gradients on the auxiliary stream), pipelined (two decoupled "
                         "kernel chains on two streams), grouped (grouped launches in both passes), stepwise (one launch per "
                         "linear and step), fused (the dependent GEMMs of a step as one launch)")
    ap.add_argument("--stage-copy", default="kernel", choices=["kernel", "memcpy"],
                    help="shard transfers by the library's copy kernel (default) or by hipMemcpyAsync device-to-device")
    ap.add_argument("--no-aux-stream", action="store_true", help="no second compute stream")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="tokens in the oracle's timed sample (0: sized for ~15 s)")
    return ap.parse_args()


def build_inputs(w, torch, dev):
    import numpy as np
    import rtp_workloads as wl
    inp = wl.make_inputs(w, seed=0)
    bf = torch.bfloat16
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev, bf)
    if w.kind == "swiglu":
        weights = [to(inp[k]) for k in ("Wg", "Wu", "Wd")]
    else:
        weights = [to(inp[k]) for k in ("W1", "W2")]
    return inp, weights, to(inp["X"]), to(inp["dY"])


class MoeUnit:
    """The expert-partitioned layer behind the same forward / backward calls as the MLP unit."""

    def __init__(self, moe, route):
        self.moe, self.route, self.compute_stream = moe, route, moe.compute_stream
        self.w_bytes, self.g_bytes = moe.w_bytes, moe.g_bytes

    def forward(self, X, Y):
        self.moe.forward(X, self.route, Y)

    def backward(self, X, dY, dX):
        self.moe.backward(dY, dX)

    def set_ablation(self, rotate=True, compute=True):
        self.moe.set_ablation(rotate, compute)

    def sync(self):
        self.moe.sync()

    def worker_bytes(self):
        return self.moe.worker_bytes()

    def close(self):
        self.moe.close()


class LinearsUnit:
    """One or several independent rotated linear layers (the fp32 single layer; the four d=2048 projections) behind
    the forward / backward calls of a unit: a pass runs every layer's N-step rotation."""

    def __init__(self, layers, torch):
        self.layers, self.torch = layers, torch            # [(name, RtpLinear, X, dY, Y, dX)]
        self.w_bytes = sum(l.ring.desc.w_bytes for _, l, *_ in layers)
        self.g_bytes = sum(l.ring.desc.g_bytes for _, l, *_ in layers)

    # The layers are independent of one another (own inputs, own streams): each one's pass is enqueued on its own
    # compute stream, ordered after the caller's stream, and the caller's stream waits for all of them at the end, so
    # that layers may share the chip (a shard GEMM of a 256-row shard is 64 tiles for 256 compute units).
    def _each(self, call):
        torch = self.torch
        cur = torch.cuda.current_stream()
        for item in self.layers:
            s = item[1].compute_stream
            if s != cur:
                s.wait_stream(cur)
            with torch.cuda.stream(s):
                call(*item)
        for item in self.layers:
            if item[1].compute_stream != cur:
                cur.wait_stream(item[1].compute_stream)

    def forward(self, X, Y):
        self._each(lambda _, l, x, dy, y, dx: l.forward(x, y))

    def backward(self, X, dY, dX):
        self._each(lambda _, l, x, dy, y, dx: l.backward(x, dy, dx))

    def set_ablation(self, rotate=True, compute=True):
        for _, l, *_ in self.layers:
            l.set_ablation(rotate, compute)

    def sync(self):
        for _, l, *_ in self.layers:
            l.sync()

    def worker_bytes(self):
        return sum(l.worker_bytes() for _, l, *_ in self.layers)

    def close(self):
        for _, l, *_ in self.layers:
            l.close()


def build_linears(w, torch, dev, aux_stream):
    import numpy as np
    import rtp_workloads as wl
    from paper_2311_01635_amd import binding as B
    from paper_2311_01635_amd.layers import RtpLinear
    inp = wl.make_inputs(w, seed=0)
    td, bd = (torch.float32, B.RTP_F32) if w.dtype == "f32" else (torch.bfloat16, B.RTP_BF16)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev, td)
    mode = {"double_buffer": B.RTP_DOUBLE_BUFFER, "inplace_staged": B.RTP_INPLACE_STAGED}[w.mode]
    mats = [("W", w.O, w.I)] if w.kind == "linear" else list(w.extra["matrices"])
    layers = []
    for (nm, O, I) in mats:
        Wn, Xn, dYn = (inp["W"], inp["X"], inp["dY"]) if w.kind == "linear" else (inp[f"W_{nm}"], inp[f"X_{I}"], inp[f"dY_{nm}"])
        layer = RtpLinear(to(Wn), w.T, w.n, 0, B.RTP_SPLIT_OUT, mode, bd, aux_stream=aux_stream)
        layers.append((nm, layer, to(Xn), to(dYn), torch.empty(w.T, O, device=dev, dtype=td), torch.empty(w.T, I, device=dev, dtype=td)))
    return inp, LinearsUnit(layers, torch)


def cpu_baseline_linears(w, inp, tokens):
    """The oracle's rotated linear layer(s), one worker, fwd+bwd, over the first `tokens` tokens (0: all of a small
    workload, else a sample sized by two short probes for roughly 15 s)."""
    import numpy as np
    import oracle as orc
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    mats = [("W", w.O, w.I)] if w.kind == "linear" else list(w.extra["matrices"])

    def run(nt):
        t0 = time.perf_counter()
        for (nm, O, I) in mats:
            Wn, Xn, dYn = (inp["W"], inp["X"], inp["dY"]) if w.kind == "linear" else (inp[f"W_{nm}"], inp[f"X_{I}"], inp[f"dY_{nm}"])
            orc.rtp_linear_out(f64(Xn[:nt]), f64(Wn), f64(dYn[:nt]), w.n, 0)
        return time.perf_counter() - t0

    if tokens <= 0 and w.flops < 1e9:
        tokens = w.T
    elif tokens <= 0:
        t16, t64 = run(16), run(64)
        per_token = max((t64 - t16) / 48.0, 1e-6)
        tokens = int(min(w.T, max(64, (15.0 - max(t16 - 16 * per_token, 0.0)) / per_token))) // 16 * 16
    dt = run(tokens)
    flops = w.flops * tokens / w.T
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"first {tokens} of {w.T} tokens, full weights, all {w.n} rotation steps fwd+bwd of "
                      f"{len(mats)} linear layer(s), {dt:.2f} s, fp64 triple loops"}


def build_moe(w, torch, dev, aux_stream):
    import numpy as np
    import rtp_workloads as wl
    from paper_2311_01635_amd import binding as B
    from paper_2311_01635_amd.layers import RtpMoe
    inp = wl.make_moe_inputs(w.T, w.I, w.O, w.O2, w.n, dtype="bf16", gated=True, seed=0, skew=w.extra["skew"],
                             w_scale=0.02, grad0=False)
    to = lambda a, t=torch.bfloat16: torch.from_numpy(np.ascontiguousarray(a)).to(dev, t)
    moe = RtpMoe([tuple(to(m) for m in ex) for ex in inp["experts"]], w.T, 0, B.RTP_ACT_SWIGLU, B.RTP_INPLACE_STAGED,
                 B.RTP_BF16, aux_stream=aux_stream)
    return inp, MoeUnit(moe, to(inp["route"], torch.int32)), to(inp["X"]), to(inp["dY"])


def cpu_baseline_moe(w, inp, tokens):
    """The oracle's expert rotation over the first `tokens` tokens (their own routing), all experts."""
    import numpy as np
    import oracle as orc
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    ex = [tuple(f64(m) for m in e) for e in inp["experts"]]

    def run(nt):
        X, dY = f64(inp["X"][:nt]), f64(inp["dY"][:nt])
        t0 = time.perf_counter()
        orc.rtp_moe(X, inp["route"][:nt], ex, dY, w.n, 0)
        return time.perf_counter() - t0

    if tokens <= 0:
        t16, t64 = run(16), run(64)
        per_token = max((t64 - t16) / 48.0, 1e-6)
        fixed = max(t16 - 16 * per_token, 0.0)
        tokens = int(min(w.T, max(64, (15.0 - fixed) / per_token))) // 16 * 16
    dt = run(tokens)
    flops = 6.0 * tokens * (2 * w.I * w.O + w.O * w.O2)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"first {tokens} of {w.T} tokens with their routing, all {w.n} experts rotating fwd+bwd, "
                      f"{dt:.1f} s, fp64 triple loops"}


def timed(torch, mlp, X, Y, dY, dX, steps, per_pass=None):
    """ms for `steps` fwd+bwd passes between one pair of HIP events on the caller's stream: a pass starts after what
    that stream holds and the stream continues after the pass (whose stage and auxiliary streams are joined into its
    compute stream when it ends), so the pair brackets all the work of every stream.  With a list in `per_pass`, an
    event between passes as well: the list receives each pass's own duration."""
    # The caller runs on the unit's own compute stream (as a training loop that owns the layer would): the pass then
    # needs no hop between the caller's stream and the layer's.  A unit of several layers has no single such stream.
    s = getattr(mlp, "compute_stream", None) or torch.cuda.current_stream()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1 if per_pass is not None else 2)]
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        marks[0].record(s)
        for i in range(steps):
            mlp.forward(X, Y)
            mlp.backward(X, dY, dX)
            if per_pass is not None:
                marks[i + 1].record(s)
        if per_pass is None:
            marks[1].record(s)
    mlp.sync()
    torch.cuda.synchronize()
    if per_pass is not None:
        per_pass.extend(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    return marks[0].elapsed_time(marks[-1])


def algorithmic_bytes(w, staging_bytes):
    """HBM bytes one fwd+bwd pass of an MLP unit has to move if every operand of every step's GEMMs is read once and
    every result written once (fp32 sums read and written each step but the first read and the last write), plus the
    staging copies.  16-bit activations and weights, fp32 gradient shards and cross-step sums."""
    gated = w.kind == "swiglu"
    P, n, T, I, O, O2 = (2 if gated else 1), w.n, w.T, w.I, w.O, w.O2
    o = O // n
    a = 2
    per_step_fwd = T * I * a + P * o * I * a + P * T * o * a + T * o * a      # X, W1_k -> pre-activations, hidden
    per_step_fwd += T * o * a + O2 * o * a                                    # hidden, W2_k -> the sum over steps
    per_step_bwd = (T * O2 * a + T * o * a + 2 * O2 * o * 4)                  # dW2: dY, hidden, G2 +=
    per_step_bwd += (T * O2 * a + O2 * o * a + P * T * o * a + P * T * o * a)   # dPre: dY, W2_k, pre-activations -> dPre
    per_step_bwd += (P * T * o * a + T * I * a + 2 * P * o * I * 4)           # dW1: dPre, X, G1 +=
    per_step_bwd += (P * T * o * a + P * o * I * a)                           # dX: dPre, W1_k -> the sum over steps
    sums = (2 * (n - 1)) * T * O2 * 4 + T * O2 * a + (2 * (n - 1)) * T * I * 4 + T * I * a
    return n * (per_step_fwd + per_step_bwd) + sums + staging_bytes


def algorithmic_bytes_linears(w, unit):
    """The same bound for independent output-partitioned linear layers: per step X, W_k and the output slice forward;
    dY slice, X and the gradient shard read and written (weight gradient), dY slice, W_k and the fp32 input-gradient sum
    read and written (input gradient) backward; plus the staging copies (each copy reads and writes its bytes)."""
    a = 4 if w.dtype == "f32" else 2
    n, T, total = w.n, w.T, 0
    mats = [("W", w.O, w.I)] if w.kind == "linear" else list(w.extra["matrices"])
    for (_, O, I) in mats:
        o = O // n
        fwd = T * I * a + o * I * a + T * o * a
        bwd = (T * o * a + T * I * a + 2 * o * I * 4) + (T * o * a + o * I * a)
        sums = (2 * (n - 1)) * T * I * 4 + T * I * a
        total += n * (fwd + bwd) + sums
    out_copied = w.dtype == "f32"              # the fp32 path copies the gradient shard out; the bf16 kernels store it home
    # gradient shard: n copies in, one copy out (the shard the pass ends on goes back to its slot when the next
    # backward pass begins), and n - 1 more out where the weight-gradient kernels do not store it home themselves
    stg = 2 * (4 * (n - 1) * unit.w_bytes + (n + 1 + (n - 1 if out_copied else 0)) * unit.g_bytes)
    return total + stg


def grad_shard_held(B, unit):
    """Whether, after a backward pass, a gradient shard is still in the worker's buffer and not in its slot."""
    if hasattr(unit, "layers"):
        rings = [l.ring.handle for _, l, *_ in unit.layers]
    elif hasattr(unit, "moe"):
        rings = [B.lib.rtp_moe_ring(unit.moe.handle)]
    else:
        rings = [B.lib.rtp_mlp_ring(unit.handle)]
    return any(B.lib.rtp_ring_resident_grad(h) >= 0 for h in rings)


def measured_traffic(workload, layout):
    """HBM bytes per launch of a GEMM kernel, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs whose
    summary is kept under profiles/ (counters cannot be read from inside this process); None if absent."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == f"{layout}_bytes_per_launch":
            return float(parts[1])
    return None


def cpu_baseline(w, inp, tokens):
    """The oracle as it stands, one worker's full rotated fwd+bwd over a token
    sample (the first `tokens` rows), timed on this host's cores.  tokens = 0:
    two short probes (16 and 64 tokens) size the sample for roughly 15 s of CPU work."""
    import numpy as np
    import oracle as orc
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    gated = w.kind == "swiglu"
    Ws = [f64(inp[k]) for k in (("Wg", "Wu", "Wd") if gated else ("W1", "W2"))]

    def run(nt):
        X, dY = f64(inp["X"][:nt]), f64(inp["dY"][:nt])
        t0 = time.perf_counter()
        if gated:
            orc.rtp_swiglu(X, *Ws, dY, w.n, 0)
        else:
            orc.rtp_mlp(X, *Ws, dY, w.n, 0)
        return time.perf_counter() - t0

    if tokens <= 0:
        t16, t64 = run(16), run(64)
        per_token = max((t64 - t16) / 48.0, 1e-6)
        fixed = max(t16 - 16 * per_token, 0.0)
        tokens = int(min(w.T, max(64, (15.0 - fixed) / per_token))) // 16 * 16
    dt = run(tokens)
    flops = 6.0 * tokens * ((2 if gated else 1) * w.I * w.O + w.O * w.O2)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"first {tokens} of {w.T} tokens, full weights, all {w.n} rotation steps fwd+bwd, "
                      f"{dt:.1f} s, fp64 triple loops"}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs one worker on one GPU (N virtual shards on the same device); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    import rtp_workloads as wl
    from paper_2311_01635_amd import binding as B
    from paper_2311_01635_amd.layers import RtpMlp

    dev = torch.device("cuda:0")
    is_moe = a.workload in wl.MOE_CONFIGS
    w = wl.MOE_CONFIGS[a.workload] if is_moe else wl.CONFIGS[a.workload]
    is_lin = w.kind in ("linear", "linears")
    X = dY = None
    if is_moe:
        inp, mlp, X, dY = build_moe(w, torch, dev, not a.no_aux_stream)
    elif is_lin:
        inp, mlp = build_linears(w, torch, dev, not a.no_aux_stream)
    else:
        inp, weights, X, dY = build_inputs(w, torch, dev)
        act = B.RTP_ACT_SWIGLU if w.kind == "swiglu" else B.RTP_ACT_GELU_ERF
        mode = {"double_buffer": B.RTP_DOUBLE_BUFFER, "inplace_staged": B.RTP_INPLACE_STAGED}[w.mode]
        mlp = RtpMlp(weights, w.T, w.n, 0, act, mode, B.RTP_BF16, stepwise=a.schedule == "stepwise",
                     grouped=a.schedule == "grouped", pipelined=a.schedule == "pipelined", fused=a.schedule == "fused", aux_stream=not a.no_aux_stream,
                     stage_memcpy=a.stage_copy == "memcpy")
    Y = dX = None
    if not is_lin:
        Y = torch.empty(w.T, w.O2, device=dev, dtype=torch.bfloat16)
        dX = torch.empty(w.T, w.I, device=dev, dtype=torch.bfloat16)
    torch.cuda.synchronize()

    timed(torch, mlp, X, Y, dY, dX, a.warmup)
    passes = []
    ms = timed(torch, mlp, X, Y, dY, dX, a.steps, per_pass=passes)
    ms_step = ms / a.steps
    passes.sort()
    tflops = w.flops / (ms_step * 1e-3) / 1e12

    # ---- the shader clock the chip sustains under this load (the MFMA peak scales with it) ----
    probe_out = torch.zeros(2, dtype=torch.int64, device=dev)
    probe_stream = torch.cuda.Stream(dev)
    torch.cuda.synchronize()
    mlp.forward(X, Y)                       # the probe starts once the load is on
    mlp.backward(X, dY, dX)
    khz = B.rtp_clock_probe(probe_stream, probe_out, int(ms_step * 1e3 * 3))
    timed(torch, mlp, X, Y, dY, dX, 5)
    torch.cuda.synchronize()
    wall, cyc = probe_out.tolist()
    clock_ghz = cyc / max(wall, 1) * khz / 1e6

    # ---- dominant kernel, instrumented repeat of the same steps --------------------
    B.rtp_prof_begin()
    timed(torch, mlp, X, Y, dY, dX, a.steps)
    prof = B.rtp_prof_end()
    dom = max(prof, key=lambda k: prof[k][1])
    launches, tot_ms, tot_flops = prof[dom]
    achieved = tot_flops / (tot_ms * 1e-3) / 1e12
    f32 = w.dtype == "f32"
    peak = PEAK_F32_VECTOR_TFLOPS if f32 else PEAK_BF16_TFLOPS
    roofline = {"bound": "alu" if f32 else "mfma",
                "kernel": "gemm_f32_kernel" if f32 else B.rtp_gemm_kernel_name({"nt": 0, "nn": 1, "tn": 2}[dom], 4),
                "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                "avg_launch_us": tot_ms * 1e3 / launches, "launches_per_step": launches / a.steps,
                "flops_per_launch": tot_flops / launches, "traffic": measured_traffic(w.name, dom),
                # launches on the compute and the auxiliary stream overlap, so a launch's duration includes the
                # time it shares the compute units with another GEMM: per-launch rates understate the kernel
                "launches_overlap": (not a.no_aux_stream),
                "per_kernel": {k: {"launches_per_step": v[0] / a.steps, "avg_us": v[1] * 1e3 / max(v[0], 1),
                                   "tflops": v[2] / max(v[1], 1e-9) / 1e9} for k, v in prof.items()}}

    # the same launches, each with the device to itself (drained before and after): what the kernel does when no
    # other GEMM and no staging copy shares the compute units and HBM with it
    k_alone = max(2, min(a.steps, 5))
    B.rtp_prof_begin(alone=True)
    timed(torch, mlp, X, Y, dY, dX, k_alone)
    prof_alone = B.rtp_prof_end()
    roofline["alone"] = {k: {"avg_us": v[1] * 1e3 / max(v[0], 1), "tflops": v[2] / max(v[1], 1e-9) / 1e9,
                             "frac": v[2] / max(v[1], 1e-9) / 1e9 / peak} for k, v in prof_alone.items()}

    # ---- how much of the shard staging hides under compute -------------------------
    overlap = None
    if not a.no_overlap and w.n > 1:
        k = max(3, a.steps // 2)
        mlp.set_ablation(rotate=False, compute=True)
        timed(torch, mlp, X, Y, dY, dX, 2)
        t_c = timed(torch, mlp, X, Y, dY, dX, k) / k
        mlp.set_ablation(rotate=True, compute=False)
        timed(torch, mlp, X, Y, dY, dX, 2)
        t_s = timed(torch, mlp, X, Y, dY, dX, k) / k
        mlp.set_ablation(rotate=True, compute=True)
        timed(torch, mlp, X, Y, dY, dX, 2)
        t_b = timed(torch, mlp, X, Y, dY, dX, k) / k
        hidden = 1.0 - max(0.0, t_b - t_c) / t_s if t_s > 0 else None
        # what the fraction covers: the copies on the stage stream.  Per pass the weights make 2(n-1) rotations (each
        # a copy out to the slot the shard travels to and a copy in from the slot it arrives in; no initial load in a
        # loop of passes: a backward pass ends on the worker's own shard); the gradient shard comes in n times by copy (n-1 rotations and the first load); the shard a pass
        # ends on is the worker's own and goes to its slot by copy only where the last kernels do not store it there.  Its other n-1 ways OUT
        # are not copies in the timed run: the weight-gradient GEMM that completes a part stores `arriving + own`
        # straight into the slot it travels to (a fused send); the staging-only run, which launches no GEMM, copies.
        n_, W_, G_ = w.n, mlp.w_bytes, mlp.g_bytes
        fused = w.dtype != "f32"                # the fp32 path copies the gradient shard out like the weights
        # the worker's own shard, on which a backward pass ends, travels no further: it is either stored straight into
        # its slot by the last step's kernels or left in the buffer and copied there when the next backward pass begins
        own_by_copy = 1 if grad_shard_held(B, mlp) else 0
        overlap = {"ms_compute_only": t_c, "ms_staging_only": t_s, "ms_both": t_b, "rotation_hidden_frac": hidden,
                   "ms_exposed": max(0.0, t_b - t_c),
                   "staged_bytes": 4 * (n_ - 1) * W_ + (n_ + own_by_copy if fused else 2 * n_) * G_, "g_out_fused": fused,
                   "own_grad_shard_written_back_by_copy": bool(own_by_copy),
                   "g_out_bytes_stored_by_gemm_epilogues": (n_ - 1) * G_ if fused else 0,
                   "staging_only_run_bytes": 4 * (n_ - 1) * W_ + 2 * n_ * G_}

    cpu = None
    if not a.no_cpu_baseline:
        cpu = (cpu_baseline_moe if is_moe else cpu_baseline_linears if is_lin else cpu_baseline)(w, inp, a.cpu_tokens)

    # ---- each matrix of a multi-layer workload on its own: K passes of that layer alone -------------
    per_matrix = None
    if is_lin and len(mlp.layers) > 1:
        per_matrix = {}
        for (nm, layer, x, dy, y, dx) in mlp.layers:
            one = LinearsUnit([(nm, layer, x, dy, y, dx)], torch)
            timed(torch, one, None, None, None, None, 2)
            ms_one = timed(torch, one, None, None, None, None, max(3, a.steps // 2)) / max(3, a.steps // 2)
            fl = 6.0 * w.T * x.shape[1] * y.shape[1]
            per_matrix[nm] = {"O": y.shape[1], "I": x.shape[1], "ms_per_pass": ms_one, "tflops": fl / (ms_one * 1e-3) / 1e12}

    hbm = None
    if is_lin:
        nbytes = algorithmic_bytes_linears(w, mlp)
        hbm = {"algorithmic_bytes_per_step": nbytes, "achieved": nbytes / (ms_step * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
               "unit": "GB/s", "frac": nbytes / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS}
    elif not is_moe:
        # staging: every copy reads and writes its bytes; per pass 2(n-1) weight rotations (out + in), the gradient
        # shard in at the start and per backward rotation (its way out is a GEMM's store, counted above) and, where
        # the last step's kernels leave the worker's own shard in the buffer, out once by copy
        stg = 2 * 4 * (w.n - 1) * mlp.w_bytes + 2 * (w.n + (1 if grad_shard_held(B, mlp) else 0)) * mlp.g_bytes
        nbytes = algorithmic_bytes(w, stg)
        hbm = {"algorithmic_bytes_per_step": nbytes, "achieved": nbytes / (ms_step * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
               "unit": "GB/s", "frac": nbytes / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS}
    out = {
        "metric": "TFLOP/s rotated-shard linear fwd+bwd per GPU", "value": tflops, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step, "ms_per_step_median": passes[len(passes) // 2],
        "ms_per_step_min": passes[0], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "T": w.T, "I": w.I, "O": w.O, "O2": w.O2, "n_shards": w.n, "mode": w.mode,
                   "grad_dtype": "f32", "flops_per_step": w.flops,
                   "schedule": "expert rotation" if is_moe else "one launch per layer and step" if is_lin else a.schedule,
                   "aux_stream": not a.no_aux_stream, "stage_copy": a.stage_copy,
                   "worker_param_bytes": mlp.worker_bytes(),
                   "table1_rtp_worker_bytes": B.rtp_table1_worker_bytes(False, mlp.w_bytes, mlp.g_bytes)},
        "per_matrix": per_matrix,
        "frac_of_bf16_mfma_peak": None if f32 else tflops / PEAK_BF16_TFLOPS,
        "sustained_clock_ghz": clock_ghz, "nominal_clock_ghz": 2.4,
        "frac_of_peak_at_sustained_clock": tflops / (peak * clock_ghz / 2.4) if clock_ghz > 0 else None,
        "roofline": roofline, "hbm_algorithmic": hbm, "overlap": overlap, "cpu_baseline": cpu,
    }
    mlp.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
