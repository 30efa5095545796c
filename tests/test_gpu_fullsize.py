"""The benchmark configurations at their full sizes, in the launch
configuration bench.py times, against the fp64 oracle on sampled outputs.

A full fp64 triple-loop oracle of these sizes would take hours, so:
  * token rows of Y, dX and the hidden activation are independent per token:
    the oracle recomputes a sample of them (first, last and random rows) with
    the whole weights;
  * rows of the weight gradients are full sums over all T tokens: the oracle
    recomputes a sample of hidden units (every shard's first and last unit
    plus random ones), i.e. rows of dW1 / dWgate / dWup and columns of dW2 /
    dWdown;
  * integers (schedule log, residency, weight store after the round trip) are
    compared exactly.
Tolerance: max-norm relative error <= 2e-2 on each sampled tensor (bf16 inputs)."""
import sys

import numpy as np
import pytest
import torch

import oracle as orc
import rtp_workloads as wl
from paper_2311_01635_amd import binding as B
from paper_2311_01635_amd.layers import RtpLinear, RtpMlp, RtpMoe

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-2


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def dev(a, dt=torch.bfloat16):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV, dt)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def relerr(got, ref):
    den = np.abs(ref).max()
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / (den if den > 0 else 1.0))


def sample_rows(total, count, rng):
    """First, last and `count` more rows, one drawn in each of `count` equal blocks: with count >= total / 128
    every 128-row tile of an output holds a sampled row, and a sampled token's row is compared over ALL its
    columns, so every output tile of Y, dX, H, the pre-activations and dPre is touched."""
    idx = {0, total - 1}
    edges = np.linspace(0, total, min(count, total) + 1).astype(int)
    idx.update(int(rng.integers(lo, hi)) for lo, hi in zip(edges[:-1], edges[1:]) if hi > lo)
    return np.array(sorted(idx))


def sample_units(O, n, extra, rng):
    """Every shard's first and last hidden unit plus `extra` more, one drawn in each of `extra` equal blocks of the
    hidden width (a sampled unit's gradient row / column is compared over its whole length)."""
    o = O // n
    idx = set()
    for k in range(n):
        idx.update((k * o, (k + 1) * o - 1))
    edges = np.linspace(0, O, extra + 1).astype(int)
    idx.update(int(rng.integers(lo, hi)) for lo, hi in zip(edges[:-1], edges[1:]) if hi > lo)
    return np.array(sorted(idx))


def _mlp_fullsize(name, n_tokens, n_extra_units, rank=0, **schedule):
    w = wl.CONFIGS[name]
    rng = np.random.default_rng(1234)
    say(f"{name}: drawing inputs")
    inp = wl.make_inputs(w, seed=0)
    gated = w.kind == "swiglu"
    names = ("Wg", "Wu", "Wd") if gated else ("W1", "W2")
    act = B.RTP_ACT_SWIGLU if gated else B.RTP_ACT_GELU_ERF
    mode = {"double_buffer": B.RTP_DOUBLE_BUFFER, "inplace_staged": B.RTP_INPLACE_STAGED}[w.mode]
    mlp = RtpMlp([dev(inp[k]) for k in names], w.T, w.n, rank, act, mode, B.RTP_BF16, **schedule)
    X, dY = dev(inp["X"]), dev(inp["dY"])
    Y = torch.full((w.T, w.O2), float("nan"), device=DEV, dtype=torch.bfloat16)
    dX = torch.full((w.T, w.I), float("nan"), device=DEV, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    say(f"{name}: GPU forward + backward, {w.n} rotation steps, mode {w.mode}, rank {rank}, schedule {schedule or 'default'}")
    for t in (mlp.preact, mlp.hidden, mlp.dpre, mlp.acc_y, mlp.acc_dx):
        t.view(torch.uint8).fill_(255)          # NaN everywhere: whatever is compared below was written by this pass
    mlp.forward(X, Y)
    mlp.backward(X, dY, dX)
    mlp.sync()
    Ws, Gs = mlp.gathered()
    for k, Wb in zip(names, Ws):
        assert torch.equal(Wb, dev(inp[k])), f"{k}: weight store changed by the round trip"
    if mode == B.RTP_INPLACE_STAGED:
        # one extra weight buffer only: never above the out-of-place row of Table 1
        assert mlp.worker_bytes() <= B.rtp_table1_worker_bytes(False, mlp.w_bytes, mlp.g_bytes)

    S = sample_rows(w.T, n_tokens, rng)
    J = sample_units(w.O, w.n, n_extra_units, rng)
    Xs, dYs = f64(inp["X"][S]), f64(inp["dY"][S])
    Xf, dYf = f64(inp["X"]), f64(inp["dY"])
    say(f"{name}: oracle on {len(S)} token rows and {len(J)} hidden units")
    if gated:
        Wg, Wu, Wd = (f64(inp[k]) for k in names)
        ref = orc.plain_swiglu(Xs, Wg, Wu, Wd, dYs)
        # full-T columns of the hidden units in J
        A = orc.gemm_nt(Xf, np.ascontiguousarray(Wg[J]), np.empty((w.T, len(J))))
        Bm = orc.gemm_nt(Xf, np.ascontiguousarray(Wu[J]), np.empty((w.T, len(J))))
        sA = orc.act(A, orc.SILU)
        H = sA * Bm
        WdJ = np.ascontiguousarray(Wd[:, J])
        dH = orc.gemm_nn(dYf, WdJ, np.empty((w.T, len(J))))
        dA = dH * Bm * orc.act_grad(A, orc.SILU)
        dB = dH * sA
        refG = {"dWg": orc.gemm_tn(dA, Xf, np.empty((len(J), w.I))), "dWu": orc.gemm_tn(dB, Xf, np.empty((len(J), w.I))),
                "dWd": orc.gemm_tn(dYf, H, np.empty((w.O2, len(J))))}
        got = {"dWg": host(Gs[0][J]), "dWu": host(Gs[1][J]), "dWd": host(Gs[2][:, J])}
    else:
        W1, W2 = (f64(inp[k]) for k in names)
        ref = orc.plain_mlp(Xs, W1, W2, dYs, orc.GELU_ERF)
        Z = orc.gemm_nt(Xf, np.ascontiguousarray(W1[J]), np.empty((w.T, len(J))))
        H = orc.act(Z, orc.GELU_ERF)
        dH = orc.gemm_nn(dYf, np.ascontiguousarray(W2[:, J]), np.empty((w.T, len(J))))
        dZ = dH * orc.act_grad(Z, orc.GELU_ERF)
        refG = {"dW1": orc.gemm_tn(dZ, Xf, np.empty((len(J), w.I))), "dW2": orc.gemm_tn(dYf, H, np.empty((w.O2, len(J))))}
        got = {"dW1": host(Gs[0][J]), "dW2": host(Gs[1][:, J])}
    got.update(Y=host(Y[S]), dX=host(dX[S]), H=host(mlp.hidden[S]))
    refs = dict(refG, Y=ref["Y"], dX=ref["dX"], H=ref["H"])
    # saved pre-activations and the gradient at them, stored shard by shard: [a_k | b_k] for the gated unit
    o = w.O // w.n
    pre, dpre = host(mlp.preact[S]), host(mlp.dpre[S])
    if gated:
        cols_a = np.concatenate([np.arange(k * 2 * o, k * 2 * o + o) for k in range(w.n)])
        got.update(A=pre[:, cols_a], Bu=pre[:, cols_a + o], dA=dpre[:, cols_a], dB=dpre[:, cols_a + o])
        refs.update(A=ref["A"], Bu=ref["B"], dA=ref["dA"], dB=ref["dB"])
    else:
        got.update(Z=pre, dZ=dpre)
        refs.update(Z=ref["Z"], dZ=ref["dZ"])
    assert torch.isfinite(Y.float()).all() and torch.isfinite(dX.float()).all(), "an output element was never written"
    errs = {k: relerr(got[k], refs[k]) for k in refs}
    say(f"{name}: max-norm relative errors {errs}")
    mlp.close()
    for k, e in errs.items():
        assert e <= TOL, (k, e)


@pytest.mark.parametrize("rank,schedule", [(0, {}), (5, dict(pipelined=True)), (3, dict(grouped=True)), (7, dict(stepwise=True)),
                                           (2, dict(aux_stream=False)), (6, dict(fused=True))])
def test_cfg4_llama7b_swiglu_fullsize(rank, schedule):
    """The headline configuration, in the launch configuration bench.py times (rank 0, default schedule) and, on other
    ranks, in every other launch schedule."""
    _mlp_fullsize("cfg4_llama7b_swiglu", n_tokens=32, n_extra_units=10, rank=rank, **schedule)


@pytest.mark.parametrize("rank,schedule", [(3, {}), (6, dict(pipelined=True)), (0, dict(stepwise=True)), (5, dict(fused=True))])
def test_cfg2_gpt2_small_mlp_fullsize(rank, schedule):
    _mlp_fullsize("cfg2_gpt2s_mlp", n_tokens=64, n_extra_units=16, rank=rank, **schedule)


@pytest.mark.parametrize("rank", [0, 9])
def test_cfg5_large_mlp_fullsize(rank):
    _mlp_fullsize("cfg5_large_mlp", n_tokens=16, n_extra_units=6, rank=rank)


def test_cfg3_d2048_projections_fullsize():
    """Four independent output-partitioned linears; the gradient shard rotates
    alongside its weight (double buffering)."""
    w = wl.CONFIGS["cfg3_d2048_proj"]
    rng = np.random.default_rng(99)
    inp = wl.make_inputs(w, seed=0)
    for (nm, O, I) in w.extra["matrices"]:
        say(f"cfg3 {nm}: [{O}, {I}], T={w.T}")
        Xn, Wn, dYn = inp[f"X_{I}"], inp[f"W_{nm}"], inp[f"dY_{nm}"]
        layer = RtpLinear(dev(Wn), w.T, w.n, 5, B.RTP_SPLIT_OUT, B.RTP_DOUBLE_BUFFER, B.RTP_BF16)
        X, dY = dev(Xn), dev(dYn)
        Y = torch.full((w.T, O), float("nan"), device=DEV, dtype=torch.bfloat16)
        dX = torch.full((w.T, I), float("nan"), device=DEV, dtype=torch.bfloat16)
        torch.cuda.synchronize()
        layer.forward(X, Y)
        layer.backward(X, dY, dX)
        layer.sync()
        Wb, G = layer.gathered()
        assert torch.equal(Wb, dev(Wn))
        tr = layer.ring.trace()
        assert [k for (kind, p, s, k, b) in tr if kind == "fwd"] == [orc.fwd_shard(5, t, w.n) for t in range(w.n)]
        assert [k for (kind, p, s, k, b) in tr if kind == "bwd"] == [orc.bwd_shard(5, t, w.n) for t in range(w.n)]
        S = sample_rows(w.T, 48, rng)
        J = sample_units(O, w.n, 16, rng)
        Wf = f64(Wn)
        refY = orc.plain_linear_fwd(f64(Xn[S]), Wf)
        refdX = orc.gemm_nn(f64(dYn[S]), Wf, np.empty((len(S), I)))
        refG = orc.gemm_tn(np.ascontiguousarray(f64(dYn)[:, J]), f64(Xn), np.empty((len(J), I)))
        errs = dict(Y=relerr(host(Y[S]), refY), dX=relerr(host(dX[S]), refdX), G=relerr(host(G[J]), refG))
        say(f"cfg3 {nm}: {errs}")
        assert torch.isfinite(Y.float()).all() and torch.isfinite(dX.float()).all()
        layer.close()
        for k, e in errs.items():
            assert e <= TOL, (nm, k, e)


@pytest.mark.parametrize("split,T,I,O,n", [(B.RTP_SPLIT_OUT, 4096, 4096, 11008, 8), (B.RTP_SPLIT_IN, 4096, 11008, 4096, 8)])
def test_integer_inputs_bit_exact_at_real_shapes(split, T, I, O, n):
    """Entries in {-2..2} at the Llama-shaped sizes: every fp32 partial sum is an
    exact integer, so the whole tensors must match a library fp64 matmul of the
    same integers bit for bit, after the same single rounding to bf16."""
    w = wl.Workload("int_full", "linear", T=T, I=I, O=O, n=n, dtype="bf16", mode="x")
    inp = wl.make_integer_inputs(w, seed=3)
    Xn, Wn, dYn = inp["X"], inp["W"], inp["dY"]
    say(f"integer-exact split={split} T={T} I={I} O={O}")
    layer = RtpLinear(dev(Wn), T, n, 2, split, B.RTP_INPLACE_STAGED, B.RTP_BF16)
    X, dY = dev(Xn), dev(dYn)
    Y = torch.empty(T, O, device=DEV, dtype=torch.bfloat16)
    dX = torch.empty(T, I, device=DEV, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    layer.forward(X, Y)
    layer.backward(X, dY, dX)
    layer.sync()
    Wb, G = layer.gathered()
    # exact integer products: a library matmul in fp64 is the plain definition here
    Xd, Wd, dYd = (torch.from_numpy(a).double() for a in (Xn, Wn, dYn))
    refY = (Xd @ Wd.T).float().to(torch.bfloat16)
    refdX = (dYd @ Wd).float().to(torch.bfloat16)
    refG = (dYd.T @ Xd).float()
    assert torch.equal(Y.cpu(), refY)
    assert torch.equal(dX.cpu(), refdX)
    assert torch.equal(G.cpu(), refG)
    assert torch.equal(Wb, dev(Wn))
    layer.close()


def test_moe_8x_swiglu_fullsize():
    """The expert-partition benchmark configuration at full size: grouping compared exactly; per
    expert a sample of its tokens (first, last, random) for Y and dX, and a sample of hidden units
    (rows of the gate/up gradients, columns of the down gradient) summed over all of its tokens."""
    w = wl.MOE_CONFIGS["moe_8x_swiglu"]
    rng = np.random.default_rng(99)
    say("moe_8x_swiglu: drawing inputs")
    inp = wl.make_moe_inputs(w.T, w.I, w.O, w.O2, w.n, dtype="bf16", gated=True, seed=0, skew=w.extra["skew"],
                             w_scale=0.02, grad0=False)
    moe = RtpMoe([tuple(dev(m) for m in ex) for ex in inp["experts"]], w.T, 0, B.RTP_ACT_SWIGLU, B.RTP_INPLACE_STAGED,
                 B.RTP_BF16)
    X, dY, route = dev(inp["X"]), dev(inp["dY"]), dev(inp["route"], torch.int32)
    Y = torch.full((w.T, w.O2), float("nan"), device=DEV, dtype=torch.bfloat16)
    dX = torch.full((w.T, w.I), float("nan"), device=DEV, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    say("moe_8x_swiglu: GPU forward + backward")
    moe.forward(X, route, Y)
    moe.backward(dY, dX)
    moe.sync()
    counts, begin, perm = orc.moe_dispatch(inp["route"], w.n, 32)
    got_counts, got_begin = moe.routing()
    assert got_counts == counts and got_begin == begin
    assert moe.perm.cpu().tolist()[:begin[w.n]] == perm
    assert torch.isfinite(Y.float()).all() and torch.isfinite(dX.float()).all(), "an output element was never written"
    assert moe.worker_bytes() <= B.rtp_table1_worker_bytes(False, moe.w_bytes, moe.g_bytes)
    Ws, Gs = moe.gathered()
    Yh, dXh = host(Y), host(dX)
    worst = {}
    for e in range(w.n):
        toks = np.array([p for p in perm[begin[e]:begin[e + 1]] if p >= 0])
        assert len(toks) == counts[e] and len(toks) > 0
        Wg, Wu, Wd = (f64(m) for m in inp["experts"][e])
        for a, b in zip(Ws[e], inp["experts"][e]):
            assert torch.equal(a, dev(b)), "weight store changed by the round trip"
        S = toks[sample_rows(len(toks), 4, rng)]
        ref = orc.plain_swiglu(f64(inp["X"][S]), Wg, Wu, Wd, f64(inp["dY"][S]))
        J = sample_rows(w.O, 3, rng)
        Xe, dYe = f64(inp["X"][toks]), f64(inp["dY"][toks])
        A = orc.gemm_nt(Xe, np.ascontiguousarray(Wg[J]), np.empty((len(toks), len(J))))
        Bm = orc.gemm_nt(Xe, np.ascontiguousarray(Wu[J]), np.empty((len(toks), len(J))))
        sA = orc.act(A, orc.SILU)
        dH = orc.gemm_nn(dYe, np.ascontiguousarray(Wd[:, J]), np.empty((len(toks), len(J))))
        refs = {"Y": ref["Y"], "dX": ref["dX"],
                "dWg": orc.gemm_tn(dH * Bm * orc.act_grad(A, orc.SILU), Xe, np.empty((len(J), w.I))),
                "dWu": orc.gemm_tn(dH * sA, Xe, np.empty((len(J), w.I))),
                "dWd": orc.gemm_tn(dYe, sA * Bm, np.empty((w.O2, len(J))))}
        got = {"Y": Yh[S], "dX": dXh[S], "dWg": host(Gs[e][0][J]), "dWu": host(Gs[e][1][J]), "dWd": host(Gs[e][2][:, J])}
        for k in refs:
            worst[k] = max(worst.get(k, 0.0), relerr(got[k], refs[k]))
        say(f"moe_8x_swiglu: expert {e}, {len(toks)} tokens, worst so far {worst}")
    moe.close()
    for k, err in worst.items():
        assert err <= TOL, (k, err)
