"""The forward step that allocates nothing (rtp_linear_fwd_noalloc) against rtp_linear_fwd and the oracle.

Same layer, same inputs, same kernels: the only difference is where the fp32 cross-step accumulator lives (a
fixed array inside the library instead of a buffer the caller brings), so the two outputs must be the same
bits; both are also held to the benchmark definition's bar against the fp64 oracle (max-norm relative error
<= 2e-2 for bf16 inputs).  Two passes run back to back through the shared array, the second on a smaller
layer, so stale content of the first would show."""
import numpy as np
import pytest
import torch

import oracle as orc
import rtp_workloads as wl
from paper_2311_01635_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL_BF16 = 2e-2


def _fwd_pass(T, I, O, n, rank, mode, seed, step_fn_name, with_acc):
    """One forward pass of an input-partitioned bf16 layer through Linear.<step_fn_name>; returns (Y, ref)."""
    w = wl.Workload("noalloc", "linear_in", T=T, I=I, O=O, n=n, dtype="bf16", mode="double_buffer", w_dist=("normal", 0.05))
    inp = wl.make_inputs(w, seed)
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    ref = orc.rtp_linear_in(f64(inp["X"]), f64(inp["W"]), f64(inp["dY"]), n, rank)["Y"]
    bf = torch.bfloat16
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV, bf)
    wb = O * (I // n) * 2
    home_w = torch.zeros(n, wb // 2, dtype=bf, device=DEV)
    B.rtp_pack_shards(home_w, wb, 0, n, B.RTP_SPLIT_IN, to(inp["W"]), O, I, I // n, B.RTP_BF16)
    home_g = torch.zeros(n, wb // 2, dtype=torch.float32, device=DEV)
    buf_w = [torch.empty(wb, dtype=torch.uint8, device=DEV) for _ in range(2)]
    buf_g = [torch.empty(2 * wb, dtype=torch.uint8, device=DEV) for _ in range(2)]
    cs, ss = torch.cuda.Stream(DEV), torch.cuda.Stream(DEV)
    ring = B.Ring(n, rank, mode, wb, 2 * wb, home_w, home_g, buf_w, buf_g, cs, ss)
    acc = torch.full((T, O), float("nan"), dtype=torch.float32, device=DEV) if with_acc else None
    lin = B.Linear(ring, T, I, O, B.RTP_SPLIT_IN, B.RTP_BF16, acc_ws=acc)
    X = to(inp["X"])
    Y = torch.full((T, O), float("nan"), dtype=bf, device=DEV)
    torch.cuda.synchronize()
    ring.begin(B.RTP_PASS_FWD)
    for t in range(n):
        if t < n - 1:
            ring.rotate_step(B.RTP_CW, t)
        getattr(lin, step_fn_name)(t, X, Y)
    ring.end()
    ring.sync()
    out = Y.float().cpu().numpy().astype(np.float64)
    ring.close()
    return out, ref


def _relerr(got, ref):
    return float(np.abs(got - ref).max() / np.abs(ref).max())


@pytest.mark.parametrize("mode", [B.RTP_DOUBLE_BUFFER, B.RTP_INPLACE_BLOCKING])
def test_two_passes_in_a_row_match_the_allocating_entry_point(mode):
    # first a layer of several tiles with ragged edges, then a smaller one: the shared array still holds
    # the first pass's sums when the second starts
    for (T, I, O, n, rank, seed) in [(520, 8 * 136, 776, 8, 3, 11), (136, 4 * 72, 264, 4, 1, 12)]:
        print(f"noalloc fwd: T={T} I={I} O={O} n={n} rank={rank} mode={mode}", flush=True)
        want, ref = _fwd_pass(T, I, O, n, rank, mode, seed, "fwd", with_acc=True)
        got, _ = _fwd_pass(T, I, O, n, rank, mode, seed, "fwd_noalloc", with_acc=False)
        assert np.isfinite(got).all()
        assert np.array_equal(got, want), "same kernels, same order of sums: the outputs must be the same bits"
        assert _relerr(want, ref) <= TOL_BF16 and _relerr(got, ref) <= TOL_BF16, (_relerr(want, ref), _relerr(got, ref))


def test_sizes_beyond_the_fixed_array_are_refused():
    T, O, I, n = 4096, 2048, 64, 2                 # fp32 [T, O] = 32 MiB, twice the array
    assert T * O * 4 > B.RTP_NOALLOC_ACC_BYTES
    wb = O * (I // n) * 2
    home_w = torch.zeros(n, wb // 2, dtype=torch.bfloat16, device=DEV)
    home_g = torch.zeros(n, wb // 2, dtype=torch.float32, device=DEV)
    buf_w = [torch.empty(wb, dtype=torch.uint8, device=DEV) for _ in range(2)]
    buf_g = [torch.empty(2 * wb, dtype=torch.uint8, device=DEV) for _ in range(2)]
    ring = B.Ring(n, 0, B.RTP_DOUBLE_BUFFER, wb, 2 * wb, home_w, home_g, buf_w, buf_g, torch.cuda.Stream(DEV), torch.cuda.Stream(DEV))
    lin = B.Linear(ring, T, I, O, B.RTP_SPLIT_IN, B.RTP_BF16)
    X = torch.zeros(T, I, dtype=torch.bfloat16, device=DEV)
    Y = torch.zeros(T, O, dtype=torch.bfloat16, device=DEV)
    ring.begin(B.RTP_PASS_FWD)
    ring.rotate_step(B.RTP_CW, 0)
    with pytest.raises(B.RtpError) as e:
        lin.fwd_noalloc(0, X, Y)
    assert e.value.status == B.RTP_ERR_SHAPE and "fixed array" in str(e.value)
    with pytest.raises(B.RtpError) as e:          # the allocating entry point, without its accumulator, says so too
        lin.fwd(0, X, Y)
    assert e.value.status == B.RTP_ERR_INVALID
    ring.abort()
    ring.sync()
    ring.close()
    # an output-partitioned layer has no accumulator in its forward pass: the variant is not for it
    ring = B.Ring(n, 0, B.RTP_DOUBLE_BUFFER, wb, 2 * wb, home_w, home_g, buf_w, buf_g, torch.cuda.Stream(DEV), torch.cuda.Stream(DEV))
    lin = B.Linear(ring, 64, O, I, B.RTP_SPLIT_OUT, B.RTP_BF16)
    with pytest.raises(B.RtpError) as e:
        lin.fwd_noalloc(0, X, Y)
    assert e.value.status == B.RTP_ERR_UNSUPPORTED
    ring.close()
