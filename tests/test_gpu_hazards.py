"""Cross-stream ordering under stretched timing.

A pass runs on three streams tied together by events.  At the timings a box happens to produce, a missing wait
can go unnoticed: the transfer it should have waited for finished long ago anyway.  Here every buffer the worker
owns is poisoned (all bits set: NaN in bf16, fp16 and fp32) before each pass, so that nothing is legally read
before it is written, and the stage stream and / or the auxiliary stream are held back by a bounded spin kernel
ahead of every transfer / every GEMM they run (rtp_ring_set_test_delay), so that they run late against the
compute stream.  The results must still be the oracle's, in every mode and every launch schedule."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle as orc
import rtp_workloads as wl
from paper_2311_01635_amd import binding as B
from paper_2311_01635_amd.layers import RtpLinear, RtpMlp, RtpMoe

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_BF16 = 2e-2
# microseconds: (stage stream, auxiliary stream, compute stream); the last case holds the COMPUTE stream back, so
# that transfers and weight-gradient kernels that did not really wait for its kernels would run ahead of them
DELAYS = [(300, 0, 0), (0, 300, 0), (300, 300, 0), (0, 0, 300)]
MODES = [B.RTP_DOUBLE_BUFFER, B.RTP_INPLACE_STAGED, B.RTP_INPLACE_BLOCKING]


def f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def dev(a, dt=torch.bfloat16):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV, dt)


def relerr(t, ref):
    g = t.detach().float().cpu().numpy().astype(np.float64)
    return float(np.abs(g - ref).max() / np.abs(ref).max())


def poison(*tensors):
    """All bits set: NaN whatever the element type (and an address nobody should follow)."""
    for t in tensors:
        if t is not None:
            t.view(torch.uint8).fill_(255)


def set_delay(ring_handle, scratch, stage_us, aux_us, compute_us=0):
    """scratch: six int64 on the device (stage, auxiliary, compute: two readings each)"""
    B.check(B.lib.rtp_ring_set_test_delay(ring_handle, B._ptr(scratch), stage_us, aux_us), "rtp_ring_set_test_delay")
    B.check(B.lib.rtp_ring_set_test_delay_compute(ring_handle, B._ptr(scratch[4:]), compute_us), "rtp_ring_set_test_delay_compute")


def spun(scratch, stage_us, aux_us, compute_us=0, blocking=False):
    """The spin kernels ran where they were asked to: they leave their wall-clock reading behind."""
    ticks = scratch.tolist()
    stage_ok = (ticks[0] > 0) == (stage_us > 0 and not blocking)      # blocking mode has no stage stream
    return stage_ok and (ticks[2] > 0) == (aux_us > 0) and (ticks[4] > 0) == (compute_us > 0)


@pytest.mark.parametrize("stage_us,aux_us,compute_us", DELAYS)
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("split", [B.RTP_SPLIT_OUT, B.RTP_SPLIT_IN])
def test_linear_layer_with_poisoned_buffers_and_late_streams(split, mode, stage_us, aux_us, compute_us):
    T, I, O, n, rank = 160, 4 * 96, 4 * 64, 4, 1
    w = wl.Workload("hz", "linear", T=T, I=I, O=O, n=n, dtype="bf16", mode="x", w_dist=("normal", 0.05))
    inp = wl.make_inputs(w, seed=71, grad0=True)
    fn = orc.rtp_linear_out if split == B.RTP_SPLIT_OUT else orc.rtp_linear_in
    ref = fn(f64(inp["X"]), f64(inp["W"]), f64(inp["dY"]), n, rank, f64(inp["G0_W"]))
    layer = RtpLinear(dev(inp["W"]), T, n, rank, split, mode, B.RTP_BF16, G0=dev(inp["G0_W"], torch.float32))
    scratch = torch.zeros(6, dtype=torch.int64, device=DEV)
    set_delay(layer.ring.handle, scratch, stage_us, aux_us, compute_us)
    X, dY = dev(inp["X"]), dev(inp["dY"])
    Y = torch.empty(T, O, device=DEV, dtype=torch.bfloat16)
    dX = torch.empty(T, I, device=DEV, dtype=torch.bfloat16)
    for p in range(2):
        print(f"linear split={split} mode={mode} delays=({stage_us},{aux_us},{compute_us}) pass {p}", flush=True)
        poison(Y, dX, layer.acc_ws, *([] if p else layer.buf_w + layer.buf_g))   # (after pass 0 the buffers hold the
        torch.cuda.synchronize()                                                 #  worker's own weight and gradient shard)
        layer.forward(X, Y)
        layer.backward(X, dY, dX)
        layer.sync()
        assert relerr(Y, ref["Y"]) <= TOL_BF16 and relerr(dX, ref["dX"]) <= TOL_BF16
    assert spun(scratch, stage_us, aux_us, compute_us, mode == B.RTP_INPLACE_BLOCKING), scratch.tolist()
    Wb, G = layer.gathered()
    assert torch.equal(Wb, dev(inp["W"]))
    two = 2.0 * ref["G"] - f64(inp["G0_W"])                                      # two passes onto what arrived
    assert relerr(G, two) <= TOL_BF16
    layer.close()


@pytest.mark.parametrize("stage_us,aux_us,compute_us", DELAYS)
@pytest.mark.parametrize("schedule", ["default", "pipelined", "grouped", "stepwise", "fused"])
@pytest.mark.parametrize("mode", MODES)
def test_mlp_unit_with_poisoned_buffers_and_late_streams(mode, schedule, stage_us, aux_us, compute_us):
    if mode == B.RTP_INPLACE_BLOCKING and schedule not in ("stepwise", "fused"):
        pytest.skip("the blocking mode runs step by step (plain or fused)")
    T, I, O, O2, n, rank = 288, 160, 4 * 128, 96, 4, 3
    w = wl.Workload("hz_mlp", "swiglu", T=T, I=I, O=O, O2=O2, n=n, dtype="bf16", mode="x", w_dist=("normal", 0.08))
    inp = wl.make_inputs(w, seed=72, grad0=True)
    names = ("Wg", "Wu", "Wd")
    ref = orc.rtp_swiglu(f64(inp["X"]), *[f64(inp[k]) for k in names], f64(inp["dY"]), n, rank,
                         *[f64(inp["G0_" + k]) for k in names])
    sched = dict(stepwise=schedule == "stepwise", grouped=schedule == "grouped", pipelined=schedule == "pipelined",
                 fused=schedule == "fused")
    mlp = RtpMlp([dev(inp[k]) for k in names], T, n, rank, B.RTP_ACT_SWIGLU, mode, B.RTP_BF16,
                 G0=[dev(inp["G0_" + k], torch.float32) for k in names], **sched)
    scratch = torch.zeros(6, dtype=torch.int64, device=DEV)
    set_delay(B.lib.rtp_mlp_ring(mlp.handle), scratch, stage_us, aux_us, compute_us)
    X, dY = dev(inp["X"]), dev(inp["dY"])
    Y = torch.empty(T, O2, device=DEV, dtype=torch.bfloat16)
    dX = torch.empty(T, I, device=DEV, dtype=torch.bfloat16)
    for p in range(2):
        print(f"mlp mode={mode} schedule={schedule} delays=({stage_us},{aux_us},{compute_us}) pass {p}", flush=True)
        poison(Y, dX, mlp.acc_y, mlp.acc_dx, mlp.preact, mlp.hidden, mlp.dpre, *([] if p else mlp.buf_w + mlp.buf_g))
        torch.cuda.synchronize()
        mlp.forward(X, Y)
        mlp.backward(X, dY, dX)
        mlp.sync()
        for key, got in (("Y", Y), ("dX", dX), ("H", mlp.hidden)):
            assert relerr(got, ref[key]) <= TOL_BF16, (key, p, relerr(got, ref[key]))
    assert spun(scratch, stage_us, aux_us, compute_us, mode == B.RTP_INPLACE_BLOCKING), scratch.tolist()
    Ws, Gs = mlp.gathered()
    assert all(torch.equal(a, dev(inp[k])) for a, k in zip(Ws, names))
    for key, k, g in zip(("dWg", "dWu", "dWd"), names, Gs):
        assert relerr(g, 2.0 * ref[key] - f64(inp["G0_" + k])) <= TOL_BF16, key
    mlp.close()


@pytest.mark.parametrize("stage_us,aux_us,compute_us", DELAYS)
def test_expert_layer_with_poisoned_buffers_and_late_streams(stage_us, aux_us, compute_us):
    n, T, rank = 4, 300, 2
    mi = wl.make_moe_inputs(T, 64, 96, 64, n, seed=73)
    ex64 = [tuple(f64(m) for m in ex) for ex in mi["experts"]]
    ref = orc.rtp_moe(f64(mi["X"]), mi["route"], ex64, f64(mi["dY"]), n, rank, G0=[tuple(f64(g) for g in ex) for ex in mi["G0"]])
    moe = RtpMoe([tuple(dev(m) for m in ex) for ex in mi["experts"]], T, rank, B.RTP_ACT_GELU_ERF,
                 G0=[tuple(dev(g, torch.float32) for g in ex) for ex in mi["G0"]])
    scratch = torch.zeros(6, dtype=torch.int64, device=DEV)
    set_delay(B.lib.rtp_moe_ring(moe.handle), scratch, stage_us, aux_us, compute_us)
    X, dY, route = dev(mi["X"]), dev(mi["dY"]), dev(mi["route"], torch.int32)
    Y = torch.empty(T, 64, device=DEV, dtype=torch.bfloat16)
    dX = torch.empty(T, 64, device=DEV, dtype=torch.bfloat16)
    print(f"moe delays=({stage_us},{aux_us},{compute_us})", flush=True)
    poison(Y, dX, moe.xp, moe.preact, moe.hidden, moe.yp, moe.dpre, moe.dxp, *moe.buf_w, *moe.buf_g)
    torch.cuda.synchronize()
    moe.forward(X, route, Y)
    moe.backward(dY, dX)
    moe.sync()
    assert relerr(Y, ref["Y"]) <= TOL_BF16 and relerr(dX, ref["dX"]) <= TOL_BF16
    assert spun(scratch, stage_us, aux_us, compute_us), scratch.tolist()
    _, Gs = moe.gathered()
    for e in range(n):
        for j in range(2):
            assert relerr(Gs[e][j], ref["G"][e][j]) <= TOL_BF16, (e, j)
    moe.close()
