"""Host-side checks that need no GPU: the library loads and exports what
include/rtp.h declares, the integer schedule is bit-exact against the oracle,
the ring's state machine orders transfers as the paper describes and rejects
calls out of sequence."""
import ctypes as C
import os
import re

import pytest

import oracle as orc
from paper_2311_01635_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "rtp.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(rtp_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 30
    lib = C.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in rtp.h but not exported"
    assert declared == set(B.SYMBOLS), "binding and header must list the same entry points"


@pytest.mark.parametrize("n", list(range(1, 65)))
def test_schedule_bit_exact_vs_oracle(n):
    for r in range(n):
        for t in range(n):
            assert B.rtp_fwd_shard(r, t, n) == orc.fwd_shard(r, t, n)
            assert B.rtp_bwd_shard(r, t, n) == orc.bwd_shard(r, t, n)


def test_schedule_rejects_bad_arguments():
    assert B.rtp_fwd_shard(0, 0, 0) == -1
    assert B.rtp_fwd_shard(4, 0, 4) == -1
    assert B.rtp_bwd_shard(0, 4, 4) == -1
    assert B.rtp_bwd_shard(-1, 0, 4) == -1
    assert B.rtp_shard_begin(0, 10, 4) == -1
    assert B.rtp_shard_begin(4, 16, 4) == -1


@pytest.mark.parametrize("dim,n", [(512, 4), (11008, 8), (28672, 16), (12, 12), (7, 1)])
def test_shard_begin_vs_oracle(dim, n):
    for k in range(n):
        assert B.rtp_shard_begin(k, dim, n) == orc.shard_rows(k, dim, n)[0]


@pytest.mark.parametrize("w,g", [(100 * 16, 100 * 16), (58720256, 117440512), (64, 32)])
def test_worker_bytes_against_table1(w, g):
    n = 16
    # Table 1 is system-wide: hand the oracle the totals and compare one worker's share
    assert B.rtp_table1_worker_bytes(False, w, g) == orc.worker_param_bytes("rtp", w * n, g * n, n)
    assert B.rtp_table1_worker_bytes(True, w, g) == orc.worker_param_bytes("rtp_inplace", w * n, g * n, n)
    assert B.rtp_worker_bytes(B.RTP_INPLACE_BLOCKING, w, g) == orc.worker_param_bytes("rtp_inplace", w * n, g * n, n)
    # one staging buffer for the weights only: never above the out-of-place row of the table
    assert B.rtp_worker_bytes(B.RTP_INPLACE_STAGED, w, g) <= B.rtp_table1_worker_bytes(False, w, g)
    assert B.rtp_worker_bytes(B.RTP_INPLACE_STAGED, w, g) == 2 * w + g
    assert B.rtp_worker_bytes(B.RTP_DOUBLE_BUFFER, w, g) == 2 * (w + g)
    assert B.rtp_worker_bytes(7, w, g) == 0


def _dry_ring(n, rank, mode, w=1024, g=2048):
    return B.Ring(n, rank, mode, w, g, flags=B.RTP_FLAG_DRY_RUN)


def _run_dry(n, rank, mode, split=B.RTP_SPLIT_OUT):
    ring = _dry_ring(n, rank, mode, w=16 * 8 * n * 4 // n * n, g=16 * 8 * n * 4 // n * n)
    lin = B.Linear(ring, 4, 8 * n if split == B.RTP_SPLIT_IN else 8, 8 * n if split == B.RTP_SPLIT_OUT else 8, split,
                   B.RTP_F32)
    ring.begin(B.RTP_PASS_FWD)
    for t in range(n):
        if t < n - 1:
            ring.rotate_step(B.RTP_CW, t)
        lin.fwd(t, None, None)
    ring.end()
    after_fwd = ring.resident()
    ring.begin(B.RTP_PASS_BWD)
    for s in range(n):
        if s < n - 1:
            ring.rotate_step(B.RTP_CCW, s)
        lin.bwd(s, None, None, None)
    ring.end()
    tr = ring.trace()
    after_bwd = ring.resident()
    ring.close()
    return tr, after_fwd, after_bwd


@pytest.mark.parametrize("mode", [B.RTP_DOUBLE_BUFFER, B.RTP_INPLACE_STAGED, B.RTP_INPLACE_BLOCKING])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 8, 16])
def test_dry_run_trace_matches_oracle_schedule(n, mode):
    """The integer record of what the ring enqueues equals the oracle's log:
    which shard each step computes on, which shard is sent and received at
    every rotation, N-1 rotations per pass, and where the worker ends."""
    import numpy as np
    X, W, dY = np.zeros((2, 3)), np.zeros((2 * n, 3)), np.zeros((2, 2 * n))
    for rank in range(n):
        tr, after_fwd, after_bwd = _run_dry(n, rank, mode)
        ref = orc.rtp_linear_out(X, W, dY, n, rank)
        assert [(s, k) for (kind, p, s, k, b) in tr if kind == "fwd"] == ref["fwd_log"]
        assert [(s, k) for (kind, p, s, k, b) in tr if kind == "bwd"] == ref["bwd_log"]
        w_out = [k for (kind, p, s, k, b) in tr if kind == "w_out" and s >= 0]
        w_in = [k for (kind, p, s, k, b) in tr if kind == "w_in" and s >= 0]
        assert w_out == ref["sent"] and w_in == ref["received"]
        assert len(w_out) == 2 * (n - 1)
        g_out = [k for (kind, p, s, k, b) in tr if kind == "g_out" and s >= 0]
        g_in = [k for (kind, p, s, k, b) in tr if kind == "g_in" and s >= 0]
        assert g_out == ref["sent"][n - 1:] and g_in == ref["received"][n - 1:], "gradients travel in the backward pass only"
        assert after_fwd == ref["resident_after_fwd"] and after_bwd == ref["resident_after_bwd"] == rank
        # the transfer that overlaps step s never targets the buffer step s computes on,
        # and lands in the buffer step s+1 computes on
        if mode != B.RTP_INPLACE_BLOCKING:
            comp = {(p, s): b for (kind, p, s, k, b) in tr if kind in ("fwd", "bwd")}
            for (kind, p, s, k, b) in tr:
                if kind == "w_in" and s >= 0:
                    assert b != comp[(p, s)] and b == comp[(p, s + 1)]


@pytest.mark.parametrize("mode", [B.RTP_DOUBLE_BUFFER, B.RTP_INPLACE_STAGED, B.RTP_INPLACE_BLOCKING])
@pytest.mark.parametrize("between", ["nothing", "flush", "abort", "forward_only", "ablation"])
def test_own_weight_shard_left_in_the_buffer_is_not_loaded_again(between, mode):
    """A backward pass ends on the worker's own shard (Design section, workflow paragraph): the next forward
    pass starts on it where it is -- same buffer, no load -- unless the store may have changed (flush), the
    ring forgot what it holds (abort, a pass without rotation) or the last pass was a forward pass."""
    n, rank = 4, 1
    ring = _dry_ring(n, rank, mode, w=16 * 8 * n * 4, g=16 * 8 * n * 4)
    lin = B.Linear(ring, 4, 8, 8 * n, B.RTP_SPLIT_OUT, B.RTP_F32)

    def fwd():
        ring.begin(B.RTP_PASS_FWD)
        for t in range(n):
            if t < n - 1:
                ring.rotate_step(B.RTP_CW, t)
            lin.fwd(t, None, None)
        ring.end()

    def bwd():
        ring.begin(B.RTP_PASS_BWD)
        for s in range(n):
            if s < n - 1:
                ring.rotate_step(B.RTP_CCW, s)
            lin.bwd(s, None, None, None)
        ring.end()

    fwd()
    first = ring.trace(clear=True)
    assert [r[3] for r in first if r[0] == "w_in" and r[2] < 0] == [rank], "first pass loads the own shard"
    bwd()
    last_bwd = [r for r in ring.trace(clear=True) if r[0] == "bwd"][-1]
    assert last_bwd[3] == rank
    if between == "flush":
        ring.flush()
    elif between == "abort":
        ring.begin(B.RTP_PASS_FWD)
        ring.abort()
    elif between == "forward_only":
        fwd()
    elif between == "ablation":
        ring.set_ablation(True, True)
    ring.trace(clear=True)
    fwd()
    tr = ring.trace(clear=True)
    loads = [r[3] for r in tr if r[0] == "w_in" and r[2] < 0]
    assert loads == ([] if between == "nothing" else [rank])
    step0 = [r for r in tr if r[0] == "fwd"][0]
    assert step0[3] == rank
    if between == "nothing":
        assert step0[4] == last_bwd[4], "step 0 computes on the buffer the backward pass ended in"
    # the schedule that follows is the same either way
    assert [r[3] for r in tr if r[0] == "fwd"] == [B.rtp_fwd_shard(rank, t, n) for t in range(n)]
    if mode != B.RTP_INPLACE_BLOCKING:
        comp = {r[2]: r[4] for r in tr if r[0] == "fwd"}
        for r in tr:
            if r[0] == "w_in" and r[2] >= 0:
                assert r[4] != comp[r[2]] and r[4] == comp[r[2] + 1]
    lin.close()
    ring.close()


@pytest.mark.parametrize("between", ["nothing", "flush", "zero_grads"])
def test_gradient_shard_left_in_the_buffer_goes_home_once(between):
    """A second backward pass first sends the worker's own gradient shard, still in its buffer from
    the first pass, to its slot; not when a flush already did, nor after the gradients were cleared."""
    n, rank = 4, 2
    ring = _dry_ring(n, rank, B.RTP_INPLACE_STAGED, w=16 * 8 * n * 4, g=16 * 8 * n * 4)
    lin = B.Linear(ring, 4, 8, 8 * n, B.RTP_SPLIT_OUT, B.RTP_F32)

    def one_pass():
        ring.begin(B.RTP_PASS_FWD)
        for t in range(n):
            if t < n - 1:
                ring.rotate_step(B.RTP_CW, t)
            lin.fwd(t, None, None)
        ring.end()
        ring.begin(B.RTP_PASS_BWD)
        for s in range(n):
            if s < n - 1:
                ring.rotate_step(B.RTP_CCW, s)
            lin.bwd(s, None, None, None)
        ring.end()

    assert ring.resident_grad() == -1
    one_pass()
    assert [r for r in ring.trace(clear=True) if r[0] == "g_out" and r[2] < 0] == [], "first pass: nothing to write back"
    assert ring.resident_grad() == rank, "the own shard's gradients are in the buffer, not yet in their slot"
    if between == "flush":
        ring.flush()
        assert [r[3] for r in ring.trace(clear=True) if r[0] == "g_out"] == [rank]
        assert ring.resident_grad() == -1
    elif between == "zero_grads":
        ring.zero_grads()
        assert ring.resident_grad() == -1
    one_pass()
    early = [r[3] for r in ring.trace(clear=True) if r[0] == "g_out" and r[2] < 0]
    assert early == ([rank] if between == "nothing" else [])
    lin.close()
    ring.begin(B.RTP_PASS_FWD)
    with pytest.raises(B.RtpError):
        ring.zero_grads()
    ring.close()


def test_state_machine_rejects_out_of_sequence_calls():
    n = 4
    ring = _dry_ring(n, 1, B.RTP_DOUBLE_BUFFER, w=16 * 32, g=16 * 32)
    lin = B.Linear(ring, 4, 8, 32, B.RTP_SPLIT_OUT, B.RTP_F32)

    def status(fn, *a):
        with pytest.raises(B.RtpError) as e:
            fn(*a)
        return e.value.status

    assert status(ring.rotate_step, B.RTP_CW, 0) == B.RTP_ERR_STATE          # no pass open
    assert status(lin.fwd, 0, None, None) == B.RTP_ERR_STATE
    assert status(ring.begin, B.RTP_PASS_BWD) == B.RTP_ERR_STATE             # backward before forward
    ring.begin(B.RTP_PASS_FWD)
    assert status(ring.begin, B.RTP_PASS_FWD) == B.RTP_ERR_STATE             # pass already open
    assert status(ring.rotate_step, B.RTP_CCW, 0) == B.RTP_ERR_STATE         # wrong direction
    assert status(ring.rotate_step, B.RTP_CW, 1) == B.RTP_ERR_STATE          # out of order
    assert status(lin.fwd, 0, None, None) == B.RTP_ERR_STATE                 # rotate first
    ring.rotate_step(B.RTP_CW, 0)
    assert status(ring.rotate_step, B.RTP_CW, 0) == B.RTP_ERR_STATE          # twice
    assert status(ring.rotate_step, B.RTP_CW, 1) == B.RTP_ERR_STATE          # linear lags behind
    assert status(lin.fwd, 1, None, None) == B.RTP_ERR_STATE                 # skips step 0
    assert status(lin.bwd, 0, None, None, None) == B.RTP_ERR_STATE           # wrong pass
    lin.fwd(0, None, None)
    assert status(lin.fwd, 1, None, None) == B.RTP_ERR_STATE                 # shard 1 not staged yet
    assert status(ring.end) == B.RTP_ERR_STATE                               # steps remain
    ring.rotate_step(B.RTP_CW, 1)
    lin.fwd(1, None, None)
    ring.rotate_step(B.RTP_CW, 2)
    lin.fwd(2, None, None)
    assert status(ring.rotate_step, B.RTP_CW, 3) == B.RTP_ERR_STATE          # only n-1 rotations
    lin.fwd(3, None, None)
    assert status(lin.fwd, 4, None, None) == B.RTP_ERR_STATE
    ring.end()
    assert ring.resident() == 2
    assert status(ring.end) == B.RTP_ERR_STATE
    ring.close()


def test_abort_is_the_way_out_of_a_failed_pass():
    """A pass that stops half-way (here: simply abandoned after two steps) leaves the ring open; rtp_ring_abort
    closes it and forgets what the worker holds, after which a forward pass starts over and the destroy calls work."""
    n = 4
    ring = _dry_ring(n, 1, B.RTP_DOUBLE_BUFFER, w=16 * 32, g=16 * 32)
    lin = B.Linear(ring, 4, 8, 32, B.RTP_SPLIT_OUT, B.RTP_F32)
    ring.abort()                                                     # idle: nothing to do
    ring.begin(B.RTP_PASS_FWD)
    ring.rotate_step(B.RTP_CW, 0)
    lin.fwd(0, None, None)
    ring.rotate_step(B.RTP_CW, 1)
    lin.fwd(1, None, None)
    for call in (ring.flush, ring.zero_grads, lambda: ring.begin(B.RTP_PASS_FWD)):
        with pytest.raises(B.RtpError) as e:
            call()
        assert e.value.status == B.RTP_ERR_STATE
    ring.abort()
    assert ring.resident() == -1
    ring.zero_grads()
    ring.flush()
    with pytest.raises(B.RtpError) as e:                             # nothing resident: a backward pass cannot start
        ring.begin(B.RTP_PASS_BWD)
    assert e.value.status == B.RTP_ERR_STATE
    ring.trace(clear=True)
    ring.begin(B.RTP_PASS_FWD)                                       # ... but a forward pass starts from step 0 again
    for t in range(n):
        if t < n - 1:
            ring.rotate_step(B.RTP_CW, t)
        lin.fwd(t, None, None)
    ring.end()
    assert [(s, k) for (kind, p, s, k, b) in ring.trace() if kind == "fwd"] == [(t, orc.fwd_shard(1, t, n)) for t in range(n)]
    ring.close()


def test_create_rejects_bad_descriptions():
    def ring_status(**kw):
        args = dict(n=4, rank=0, mode=B.RTP_DOUBLE_BUFFER, w_bytes=64, g_bytes=64, flags=B.RTP_FLAG_DRY_RUN)
        args.update(kw)
        try:
            B.Ring(**args).close()
            return B.RTP_OK
        except B.RtpError as e:
            return e.status

    assert ring_status() == B.RTP_OK
    assert ring_status(n=0) == B.RTP_ERR_SHAPE
    assert ring_status(rank=4) == B.RTP_ERR_SHAPE
    assert ring_status(w_bytes=24) == B.RTP_ERR_SHAPE
    assert ring_status(mode=9) == B.RTP_ERR_INVALID
    assert ring_status(flags=0) == B.RTP_ERR_INVALID           # real run with null device buffers

    ring = _dry_ring(4, 0, B.RTP_DOUBLE_BUFFER, w=16 * 1024, g=32 * 1024)

    def lin_status(**kw):
        args = dict(T=8, I=64, O=64, split=B.RTP_SPLIT_OUT, dtype=B.RTP_BF16)
        args.update(kw)
        try:
            B.Linear(ring, **args).close()
            return B.RTP_OK
        except B.RtpError as e:
            return e.status

    assert lin_status() == B.RTP_OK
    assert lin_status(O=66) == B.RTP_ERR_SHAPE                 # 4 does not divide 66
    assert lin_status(O=48) == B.RTP_ERR_SHAPE                 # shard width 12 is not a multiple of 8
    assert lin_status(I=60) == B.RTP_ERR_SHAPE
    assert lin_status(I=0) == B.RTP_ERR_SHAPE
    assert lin_status(dtype=B.RTP_F16) == B.RTP_ERR_UNSUPPORTED        # fp16: shard width 16 is not a multiple of 32
    assert lin_status(dtype=B.RTP_F16, T=32, I=64, O=128) == B.RTP_OK
    assert lin_status(dtype=B.RTP_F16, T=40, I=64, O=128) == B.RTP_ERR_UNSUPPORTED
    assert lin_status(grad_dtype=B.RTP_BF16) == B.RTP_ERR_UNSUPPORTED
    assert lin_status(O=4096) == B.RTP_ERR_SHAPE               # shard larger than the slot
    assert lin_status(w_offset=8) == B.RTP_ERR_SHAPE
    assert lin_status(split=5) == B.RTP_ERR_INVALID
    assert lin_status(has_bias=True) == B.RTP_OK
    assert lin_status(has_bias=True, split=B.RTP_SPLIT_IN) == B.RTP_OK                # bias spread over the shards in pieces
    assert lin_status(O=512) == B.RTP_OK                                               # 128 x 64 rows fill the slot exactly
    assert lin_status(has_bias=True, O=512) == B.RTP_ERR_SHAPE                         # ... so the bias entries do not fit
    assert lin_status(dtype=B.RTP_F32, O=12, I=3) == B.RTP_OK  # fp32 has no alignment rule
    ring.close()
    assert B.lib.rtp_status_str(B.RTP_ERR_STATE) == b"RTP_ERR_STATE"


def test_mlp_slot_sizes():
    d = B.rtp_mlp_desc()
    d.T, d.I, d.O, d.O2, d.n, d.dtype, d.act = 4096, 4096, 11008, 4096, 8, B.RTP_BF16, B.RTP_ACT_SWIGLU
    assert B.lib.rtp_mlp_slot_w_bytes(C.byref(d)) == 3 * 1376 * 4096 * 2
    assert B.lib.rtp_mlp_slot_g_bytes(C.byref(d)) == 3 * 1376 * 4096 * 4
    d.act, d.I, d.O, d.O2, d.n, d.T = B.RTP_ACT_GELU_ERF, 8192, 28672, 8192, 16, 2048
    w, g = B.lib.rtp_mlp_slot_w_bytes(C.byref(d)), B.lib.rtp_mlp_slot_g_bytes(C.byref(d))
    assert (w, g) == (58720256, 117440512)
    # a hidden width n does not divide: n shards of the aligned width that covers it
    d2 = B.rtp_mlp_desc()
    d2.T, d2.I, d2.O, d2.O2, d2.n, d2.dtype, d2.act = 64, 64, 232, 64, 6, B.RTP_BF16, B.RTP_ACT_SWIGLU
    assert B.lib.rtp_mlp_hidden_width(C.byref(d2)) == 240
    assert B.lib.rtp_mlp_slot_w_bytes(C.byref(d2)) == (2 * 40 * 64 + 64 * 40) * 2
    d2.O = 200                                           # 5 shards of 40 would cover it: the last shard would be empty
    assert B.lib.rtp_mlp_hidden_width(C.byref(d2)) == -1 and B.lib.rtp_mlp_slot_w_bytes(C.byref(d2)) == 0
    assert B.lib.rtp_mlp_hidden_width(C.byref(d)) == 28672
    # the large config's footprint against the table's per-worker bound
    assert B.rtp_worker_bytes(B.RTP_INPLACE_STAGED, w, g) == 234881024
    assert B.rtp_table1_worker_bytes(False, w, g) == orc.worker_param_bytes("rtp", 939524096, 1879048192, 16)


def test_build_script_loads_without_the_library():
    """build() must work on a tree that holds no built library yet: the build script is loaded by
    path (the package itself refuses to import without librtp.so) and names sources that exist."""
    import os

    import __graft_entry__ as entry
    root = os.path.dirname(os.path.abspath(entry.__file__))
    mod = entry._load_by_path("_rtp_lib_build_test", os.path.join(root, "paper_2311_01635_amd", "build.py"))
    for src in mod.SOURCES:
        assert os.path.exists(os.path.join(mod.CSRC, src)), src
    assert "paper_2311_01635_amd" not in open(entry.__file__).read().split("def build()")[1].split("lib_build.build")[0].replace(
        '"paper_2311_01635_amd"', ""), "build() imports the package before building it"


def test_shard_width_with_padding():
    """Equal shards; when n does not divide the dimension the width is rounded up to the element
    alignment of the dtype and the last shard is partly filled, never empty."""
    w = B.lib.rtp_shard_width
    assert w(512, 4, B.RTP_BF16) == 128 and w(512, 4, B.RTP_F32) == 128
    assert w(520, 3, B.RTP_BF16) == 176            # ceil(520/3) = 174 -> 176; shards 176, 176, 168
    assert w(50, 3, B.RTP_F32) == 17               # 17, 17, 16
    assert w(1056, 5, B.RTP_F16) == 224            # ceil = 212 -> 224; last shard 1056 - 896 = 160
    assert w(42, 4, B.RTP_BF16) == -1              # width 16: shards 16, 16, 10, 0 -- the last would be empty
    assert w(40, 4, B.RTP_BF16) == 10              # n divides: no padding (a bf16 layer then fails on alignment)
    assert w(0, 4, B.RTP_BF16) == -1 and w(64, 0, B.RTP_BF16) == -1
    for dim, n, dt, al in ((520, 3, B.RTP_BF16, 8), (1000, 7, B.RTP_F32, 1), (4000, 6, B.RTP_BF16, 8)):
        o = w(dim, n, dt)
        assert o % al == 0 and (n - 1) * o < dim <= n * o and o - al < -(-dim // n) <= o


def test_padded_linear_descriptions():
    ring = _dry_ring(3, 0, B.RTP_DOUBLE_BUFFER, w=176 * 64 * 2, g=176 * 64 * 4)
    ok = B.Linear(ring, T=8, I=64, O=520, split=B.RTP_SPLIT_OUT, dtype=B.RTP_BF16)      # shards of 176 rows, padded
    ok.close()
    ok = B.Linear(ring, T=8, I=64, O=520, split=B.RTP_SPLIT_OUT, dtype=B.RTP_BF16, act=B.RTP_ACT_GELU_ERF)   # also with an activation
    ok.close()
    with pytest.raises(B.RtpError) as e:                                                  # but not a gated one: the unit pads itself
        B.Linear(ring, T=8, I=64, O=520, split=B.RTP_SPLIT_OUT, dtype=B.RTP_BF16, act=B.RTP_ACT_SWIGLU)
    assert e.value.status == B.RTP_ERR_SHAPE
    with pytest.raises(B.RtpError) as e:                                                  # padded shard larger than the slot
        B.Linear(ring, T=8, I=64, O=536, split=B.RTP_SPLIT_OUT, dtype=B.RTP_BF16)
    assert e.value.status == B.RTP_ERR_SHAPE
    ring.close()


# ------------------------------------------------------ expert partition --

def test_moe_padded_rows_bound_every_routing():
    """The grouped workspace holds any routing: groups padded to 32 rows never exceed it, and the
    bound is attained."""
    import numpy as np
    rng = np.random.default_rng(0)
    assert B.lib.rtp_moe_padded_rows(-1, 4) == -1 and B.lib.rtp_moe_padded_rows(10, 0) == -1
    for n in (1, 2, 5, 8, 64):
        for T in (0, 1, 31, 32, 33, 200, 4096):
            cap = B.lib.rtp_moe_padded_rows(T, n)
            assert cap % 32 == 0
            worst = 0
            for trial in range(20):
                route = rng.integers(0, n, T)
                _, begin, _ = orc.moe_dispatch(route, n, 32)
                worst = max(worst, begin[n])
            # the adversarial routing: one token over a multiple of 32 on as many experts as possible
            c = [0] * n
            left = T
            for e in range(n - 1):
                if left >= 1:
                    c[e] = 1
                    left -= 1
            c[n - 1] = left
            worst = max(worst, sum((x + 31) // 32 * 32 for x in c))
            assert worst <= cap
    assert B.lib.rtp_moe_padded_rows(33, 2) == 96 and sum((x + 31) // 32 * 32 for x in (1, 32)) == 64


def _moe_desc(**kw):
    import ctypes as C
    d = B.rtp_moe_desc()
    d.T, d.I, d.O, d.O2, d.n, d.rank = 128, 64, 96, 64, 4, 0
    d.mode, d.dtype, d.act, d.flags = B.RTP_INPLACE_STAGED, B.RTP_BF16, B.RTP_ACT_GELU_ERF, 0
    fake = 0x1000
    for name in ("home_w_dev", "home_g_dev", "xp_dev", "preact_dev", "hidden_dev", "yp_dev", "dpre_dev", "dxp_dev",
                 "perm_dev", "counts_dev", "compute_stream", "stage_stream"):
        fake += 0x1000
        setattr(d, name, fake)
    d.buf_w_dev[0], d.buf_w_dev[1], d.buf_g_dev[0] = 0x100000, 0x200000, 0x300000
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_moe_descriptions():
    import ctypes as C
    d = _moe_desc()
    assert B.lib.rtp_moe_slot_w_bytes(C.byref(d)) == (96 * 64 + 64 * 96) * 2
    assert B.lib.rtp_moe_slot_g_bytes(C.byref(d)) == (96 * 64 + 64 * 96) * 4
    g = _moe_desc(act=B.RTP_ACT_SWIGLU)
    assert B.lib.rtp_moe_slot_w_bytes(C.byref(g)) == (2 * 96 * 64 + 64 * 96) * 2, "a gated expert holds gate and up"
    h = C.c_void_p()
    assert B.lib.rtp_moe_create(C.byref(h), C.byref(d)) == B.RTP_OK      # validation and bookkeeping only: no GPU call
    assert B.lib.rtp_moe_ring(h) is not None
    assert B.lib.rtp_moe_bwd(h, 0x1000, 0x1000) == B.RTP_ERR_STATE, "backward needs a forward's routing"
    assert B.lib.rtp_moe_routing(h, None, None) == B.RTP_ERR_STATE
    assert B.lib.rtp_moe_destroy(h) == B.RTP_OK
    bad = [
        (dict(flags=B.RTP_FLAG_DRY_RUN), B.RTP_ERR_UNSUPPORTED),
        (dict(act=B.RTP_ACT_NONE), B.RTP_ERR_INVALID),
        (dict(dtype=B.RTP_F32), B.RTP_ERR_UNSUPPORTED),
        (dict(n=65), B.RTP_ERR_SHAPE),
        (dict(n=0), B.RTP_ERR_SHAPE),
        (dict(I=60), B.RTP_ERR_SHAPE),
        (dict(O2=0), B.RTP_ERR_SHAPE),
        (dict(dtype=B.RTP_F16, O=72), B.RTP_ERR_UNSUPPORTED),
        (dict(perm_dev=None), B.RTP_ERR_INVALID),
        (dict(rank=4), B.RTP_ERR_SHAPE),
        (dict(stage_stream=_moe_desc().compute_stream), B.RTP_ERR_INVALID),
    ]
    for kw, want in bad:
        h = C.c_void_p()
        assert B.lib.rtp_moe_create(C.byref(h), C.byref(_moe_desc(**kw))) == want, kw
        assert not h.value


def test_bias_piece_width_and_slot_sizes():
    """Piece of an input-partitioned layer's bias: ceil(O / n) rounded up to 16 bytes; the shard sizes
    count it; an MLP unit with biases = the two linears' shards back to back."""
    assert B.lib.rtp_bias_piece_width(768, 8, B.RTP_BF16) == 96
    assert B.lib.rtp_bias_piece_width(100, 8, B.RTP_BF16) == 16        # ceil = 13 -> 16
    assert B.lib.rtp_bias_piece_width(100, 8, B.RTP_F32) == 16         # 13 -> 16 (multiples of 4)
    assert B.lib.rtp_bias_piece_width(10, 8, B.RTP_F32) == 4           # ceil = 2 -> 4
    assert B.lib.rtp_bias_piece_width(0, 8, B.RTP_F32) == -1 and B.lib.rtp_bias_piece_width(8, 0, B.RTP_F32) == -1
    for O in (8, 100, 768, 4096):
        for n in (1, 3, 8, 16):
            p = B.lib.rtp_bias_piece_width(O, n, B.RTP_BF16)
            pieces = orc.bias_pieces(O, n)
            assert p >= max(hi - lo for lo, hi in pieces) and n * p >= O and p % 8 == 0
    d = B.rtp_linear_desc()
    d.T, d.I, d.O, d.split, d.dtype, d.grad_dtype, d.has_bias = 64, 256, 100, B.RTP_SPLIT_IN, B.RTP_BF16, B.RTP_F32, 1
    assert B.lib.rtp_linear_shard_w_bytes(C.byref(d), 8) == (100 * 32 + 16) * 2
    assert B.lib.rtp_linear_shard_g_bytes(C.byref(d), 8) == (100 * 32 + 16) * 4
    m = B.rtp_mlp_desc()
    m.T, m.I, m.O, m.O2, m.n, m.dtype, m.act = 64, 128, 512, 100, 8, B.RTP_BF16, B.RTP_ACT_GELU_ERF
    plain = B.lib.rtp_mlp_slot_w_bytes(C.byref(m))
    assert plain == (512 * 128 + 100 * 512) // 8 * 2
    m.has_bias = 1
    assert B.lib.rtp_mlp_slot_w_bytes(C.byref(m)) == plain + (64 + 16) * 2
    assert B.lib.rtp_mlp_slot_g_bytes(C.byref(m)) == 2 * (plain + (64 + 16) * 2)


def test_header_is_plain_c():
    """The boundary is a C ABI: the header compiles as C99 and as C++ with no torch or HIP type in sight."""
    import shutil
    import subprocess
    hdr = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "rtp.h")
    if shutil.which("gcc") is None:
        pytest.skip("no host C compiler")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", hdr], check=True)
    text = open(hdr).read()
    assert "torch" not in text.lower() and "hipStream_t " not in text.replace("/* hipStream_t", "")


def test_shard_layout_calls_validate_before_they_launch():
    """rtp_pack_shards / rtp_unpack_shards reject bad descriptions on the host (no kernel is launched)."""
    import ctypes as C
    p = C.c_void_p(4096)     # never dereferenced: every call below fails validation first

    def st(home, slot, off, n, split, W, O, I, w, dt):
        return B.lib.rtp_pack_shards(home, slot, off, n, split, W, O, I, w, dt, None)

    assert st(None, 1024, 0, 4, B.RTP_SPLIT_OUT, p, 8, 8, 2, B.RTP_BF16) == B.RTP_ERR_INVALID
    assert st(p, 1024, 0, 4, B.RTP_SPLIT_OUT, None, 8, 8, 2, B.RTP_BF16) == B.RTP_ERR_INVALID
    assert st(p, 1024, 0, 4, 7, p, 8, 8, 2, B.RTP_BF16) == B.RTP_ERR_INVALID
    assert st(p, 1024, 0, 4, B.RTP_SPLIT_OUT, p, 8, 8, 2, 9) == B.RTP_ERR_INVALID
    assert st(p, 1024, 0, 0, B.RTP_SPLIT_OUT, p, 8, 8, 2, B.RTP_BF16) == B.RTP_ERR_SHAPE       # n < 1
    assert st(p, 1024, 0, 4, B.RTP_SPLIT_OUT, p, 9, 8, 2, B.RTP_BF16) == B.RTP_ERR_SHAPE       # 4 x 2 rows do not cover 9
    assert st(p, 1024, 0, 4, B.RTP_SPLIT_IN, p, 8, 9, 2, B.RTP_BF16) == B.RTP_ERR_SHAPE
    assert st(p, 31, 0, 4, B.RTP_SPLIT_OUT, p, 8, 8, 2, B.RTP_BF16) == B.RTP_ERR_SHAPE         # part of 32 bytes, slot of 31
    assert st(p, 1024, 1000, 4, B.RTP_SPLIT_OUT, p, 8, 8, 2, B.RTP_BF16) == B.RTP_ERR_SHAPE    # offset pushes it out
    assert st(p, 1024, 1, 4, B.RTP_SPLIT_OUT, p, 8, 8, 2, B.RTP_BF16) == B.RTP_ERR_SHAPE       # offset not a whole element
    assert B.lib.rtp_unpack_shards(p, None, 1024, 0, 4, B.RTP_SPLIT_OUT, 8, 8, 2, B.RTP_BF16, None) == B.RTP_ERR_INVALID
    assert b"rtp_unpack_shards" in B.lib.rtp_last_error()
