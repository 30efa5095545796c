"""ctypes binding of librtp.so -- argument marshalling only.

Every name mirrors include/rtp.h.  Torch is used for device memory and
streams; every step of the path runs in the library's kernels.  Loading fails
loudly when the shared library has not been built: there is no fallback.
"""
import ctypes as C
import os

# torch first: librtp.so must bind to the HIP runtime torch has loaded.  Loaded the other way round,
# the library pulls in the system's copy and torch's tensors then live in a different runtime
# (every HIP call of the library fails with "no ROCm-capable device").
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librtp.so")

# enums (include/rtp.h)
RTP_OK, RTP_ERR_INVALID, RTP_ERR_SHAPE, RTP_ERR_STATE, RTP_ERR_UNSUPPORTED, RTP_ERR_HIP = range(6)
RTP_F32, RTP_BF16, RTP_F16 = 0, 1, 2
RTP_SPLIT_OUT, RTP_SPLIT_IN = 0, 1
RTP_DOUBLE_BUFFER, RTP_INPLACE_STAGED, RTP_INPLACE_BLOCKING = 0, 1, 2
RTP_ACT_NONE, RTP_ACT_GELU_ERF, RTP_ACT_GELU_TANH, RTP_ACT_SWIGLU = 0, 1, 2, 3
RTP_PASS_IDLE, RTP_PASS_FWD, RTP_PASS_BWD = 0, 1, 2
RTP_CW, RTP_CCW = 1, -1
RTP_FLAG_DRY_RUN = 1
RTP_FLAG_STEPWISE = 2
RTP_FLAG_GROUPED = 4
RTP_FLAG_PIPELINED = 8
RTP_FLAG_STAGE_MEMCPY = 16
RTP_FLAG_FUSED_STEP = 32
RTP_NOALLOC_ACC_BYTES = 16 << 20
LAYOUT_NT, LAYOUT_NN, LAYOUT_TN = 0, 1, 2

TRACE_KINDS = {1: "fwd", 2: "bwd", 3: "w_in", 4: "w_out", 5: "g_in", 6: "g_out"}


class rtp_ring_desc(C.Structure):
    _fields_ = [("n", C.c_int), ("rank", C.c_int), ("mode", C.c_int), ("flags", C.c_uint),
                ("w_bytes", C.c_size_t), ("g_bytes", C.c_size_t),
                ("home_w_dev", C.c_void_p), ("home_g_dev", C.c_void_p),
                ("buf_w_dev", C.c_void_p * 2), ("buf_g_dev", C.c_void_p * 2),
                ("compute_stream", C.c_void_p), ("stage_stream", C.c_void_p), ("aux_stream", C.c_void_p)]


class rtp_linear_desc(C.Structure):
    _fields_ = [("T", C.c_int64), ("I", C.c_int64), ("O", C.c_int64),
                ("split", C.c_int), ("dtype", C.c_int), ("grad_dtype", C.c_int), ("act", C.c_int),
                ("w_offset", C.c_size_t), ("g_offset", C.c_size_t),
                ("preact_dev", C.c_void_p), ("acc_ws_dev", C.c_void_p), ("has_bias", C.c_int)]


class rtp_mlp_desc(C.Structure):
    _fields_ = [("T", C.c_int64), ("I", C.c_int64), ("O", C.c_int64), ("O2", C.c_int64),
                ("n", C.c_int), ("rank", C.c_int), ("mode", C.c_int), ("dtype", C.c_int),
                ("act", C.c_int), ("flags", C.c_uint),
                ("home_w_dev", C.c_void_p), ("home_g_dev", C.c_void_p),
                ("buf_w_dev", C.c_void_p * 2), ("buf_g_dev", C.c_void_p * 2),
                ("preact_dev", C.c_void_p), ("hidden_dev", C.c_void_p), ("dpre_dev", C.c_void_p),
                ("acc_y_dev", C.c_void_p), ("acc_dx_dev", C.c_void_p),
                ("compute_stream", C.c_void_p), ("stage_stream", C.c_void_p), ("aux_stream", C.c_void_p),
                ("step_sync_dev", C.c_void_p), ("has_bias", C.c_int)]


class rtp_moe_desc(C.Structure):
    _fields_ = [("T", C.c_int64), ("I", C.c_int64), ("O", C.c_int64), ("O2", C.c_int64),
                ("n", C.c_int), ("rank", C.c_int), ("mode", C.c_int), ("dtype", C.c_int),
                ("act", C.c_int), ("flags", C.c_uint),
                ("home_w_dev", C.c_void_p), ("home_g_dev", C.c_void_p),
                ("buf_w_dev", C.c_void_p * 2), ("buf_g_dev", C.c_void_p * 2),
                ("xp_dev", C.c_void_p), ("preact_dev", C.c_void_p), ("hidden_dev", C.c_void_p),
                ("yp_dev", C.c_void_p), ("dpre_dev", C.c_void_p), ("dxp_dev", C.c_void_p),
                ("perm_dev", C.c_void_p), ("counts_dev", C.c_void_p),
                ("compute_stream", C.c_void_p), ("stage_stream", C.c_void_p), ("aux_stream", C.c_void_p)]


class rtp_prof_result(C.Structure):
    _fields_ = [("launches", C.c_int64), ("total_ms", C.c_double), ("total_flops", C.c_double)]


class rtp_trace_rec(C.Structure):
    _fields_ = [("kind", C.c_int), ("pass_", C.c_int), ("step", C.c_int), ("shard", C.c_int), ("buffer", C.c_int)]


# every symbol include/rtp.h declares: name -> (restype, argtypes)
_P = C.c_void_p
SYMBOLS = {
    "rtp_fwd_shard": (C.c_int, [C.c_int, C.c_int, C.c_int]),
    "rtp_bwd_shard": (C.c_int, [C.c_int, C.c_int, C.c_int]),
    "rtp_shard_begin": (C.c_int64, [C.c_int, C.c_int64, C.c_int]),
    "rtp_shard_width": (C.c_int64, [C.c_int64, C.c_int, C.c_int]),
    "rtp_bias_piece_width": (C.c_int64, [C.c_int64, C.c_int, C.c_int]),
    "rtp_linear_shard_w_bytes": (C.c_size_t, [C.POINTER(rtp_linear_desc), C.c_int]),
    "rtp_linear_shard_g_bytes": (C.c_size_t, [C.POINTER(rtp_linear_desc), C.c_int]),
    "rtp_worker_bytes": (C.c_size_t, [C.c_int, C.c_size_t, C.c_size_t]),
    "rtp_table1_worker_bytes": (C.c_size_t, [C.c_int, C.c_size_t, C.c_size_t]),
    "rtp_pack_shards": (C.c_int, [_P, C.c_size_t, C.c_size_t, C.c_int, C.c_int, _P, C.c_int64, C.c_int64, C.c_int64, C.c_int, _P]),
    "rtp_unpack_shards": (C.c_int, [_P, _P, C.c_size_t, C.c_size_t, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int, _P]),
    "rtp_status_str": (C.c_char_p, [C.c_int]),
    "rtp_prof_begin_alone": (C.c_int, [C.c_int]),
    "rtp_clock_probe": (C.c_int, [_P, _P, C.c_int64, C.POINTER(C.c_int)]),
    "rtp_last_error": (C.c_char_p, []),
    "rtp_ring_create": (C.c_int, [C.POINTER(_P), C.POINTER(rtp_ring_desc)]),
    "rtp_ring_destroy": (C.c_int, [_P]),
    "rtp_ring_begin": (C.c_int, [_P, C.c_int]),
    "rtp_ring_seek_bwd_start": (C.c_int, [_P]),
    "rtp_rotate_step": (C.c_int, [_P, C.c_int, C.c_int]),
    "rtp_ring_end": (C.c_int, [_P]),
    "rtp_ring_abort": (C.c_int, [_P]),
    "rtp_ring_set_test_delay": (C.c_int, [_P, _P, C.c_int64, C.c_int64]),
    "rtp_ring_set_test_delay_compute": (C.c_int, [_P, _P, C.c_int64]),
    "rtp_ring_set_ablation": (C.c_int, [_P, C.c_int, C.c_int]),
    "rtp_ring_flush": (C.c_int, [_P]),
    "rtp_ring_zero_grads": (C.c_int, [_P]),
    "rtp_ring_sync": (C.c_int, [_P]),
    "rtp_ring_resident": (C.c_int, [_P]),
    "rtp_ring_resident_grad": (C.c_int, [_P]),
    "rtp_ring_trace": (C.c_int64, [_P, C.POINTER(rtp_trace_rec), C.c_int64, C.c_int]),
    "rtp_linear_create": (C.c_int, [C.POINTER(_P), _P, C.POINTER(rtp_linear_desc)]),
    "rtp_linear_destroy": (C.c_int, [_P]),
    "rtp_linear_fwd": (C.c_int, [_P, C.c_int, _P, _P]),
    "rtp_linear_bwd": (C.c_int, [_P, C.c_int, _P, _P, _P]),
    "rtp_linear_fwd_noalloc": (C.c_int, [_P, C.c_int, _P, _P]),
    "rtp_mlp_hidden_width": (C.c_int64, [C.POINTER(rtp_mlp_desc)]),
    "rtp_mlp_step_sync_bytes": (C.c_size_t, [C.POINTER(rtp_mlp_desc)]),
    "rtp_mlp_slot_w_bytes": (C.c_size_t, [C.POINTER(rtp_mlp_desc)]),
    "rtp_mlp_slot_g_bytes": (C.c_size_t, [C.POINTER(rtp_mlp_desc)]),
    "rtp_mlp_create": (C.c_int, [C.POINTER(_P), C.POINTER(rtp_mlp_desc)]),
    "rtp_mlp_destroy": (C.c_int, [_P]),
    "rtp_mlp_fwd": (C.c_int, [_P, _P, _P]),
    "rtp_mlp_bwd": (C.c_int, [_P, _P, _P, _P]),
    "rtp_mlp_set_ablation": (C.c_int, [_P, C.c_int, C.c_int]),
    "rtp_mlp_flush": (C.c_int, [_P]),
    "rtp_mlp_sync": (C.c_int, [_P]),
    "rtp_mlp_ring": (_P, [_P]),
    "rtp_moe_padded_rows": (C.c_int64, [C.c_int64, C.c_int]),
    "rtp_moe_slot_w_bytes": (C.c_size_t, [C.POINTER(rtp_moe_desc)]),
    "rtp_moe_slot_g_bytes": (C.c_size_t, [C.POINTER(rtp_moe_desc)]),
    "rtp_moe_create": (C.c_int, [C.POINTER(_P), C.POINTER(rtp_moe_desc)]),
    "rtp_moe_destroy": (C.c_int, [_P]),
    "rtp_moe_fwd": (C.c_int, [_P, _P, _P, _P]),
    "rtp_moe_bwd": (C.c_int, [_P, _P, _P]),
    "rtp_moe_routing": (C.c_int, [_P, C.POINTER(C.c_int32), C.POINTER(C.c_int64)]),
    "rtp_moe_flush": (C.c_int, [_P]),
    "rtp_moe_set_ablation": (C.c_int, [_P, C.c_int, C.c_int]),
    "rtp_moe_sync": (C.c_int, [_P]),
    "rtp_moe_ring": (_P, [_P]),
    "rtp_gemm": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, _P, C.c_int64, _P, C.c_int64, _P, C.c_int64,
                           C.c_int64, C.c_int64, C.c_int64, C.c_int, _P]),
    "rtp_gemm_kernel_name": (C.c_char_p, [C.c_int, C.c_int]),
    "rtp_prof_begin": (C.c_int, []),
    "rtp_prof_end": (C.c_int, [C.POINTER(rtp_prof_result)]),
}


def load_library(path: str = LIB_PATH):
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python paper_2311_01635_amd/build.py` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(path)
    for name, (res, args) in SYMBOLS.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


lib = load_library()


class RtpError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib.rtp_last_error().decode()
        super().__init__(f"{where}: {lib.rtp_status_str(status).decode()}: {msg}")


def check(status, where=""):
    if status != RTP_OK:
        raise RtpError(status, where)


# plain helpers with the header's names
def rtp_fwd_shard(rank, step, n):
    return lib.rtp_fwd_shard(rank, step, n)


def rtp_bwd_shard(rank, step, n):
    return lib.rtp_bwd_shard(rank, step, n)


def rtp_shard_begin(k, dim, n):
    return lib.rtp_shard_begin(k, dim, n)


def rtp_worker_bytes(mode, w, g):
    return lib.rtp_worker_bytes(mode, w, g)


def rtp_table1_worker_bytes(inplace, w, g):
    return lib.rtp_table1_worker_bytes(int(inplace), w, g)


def _ptr(t):
    """Device (or host) address of a torch tensor, or None."""
    if t is None:
        return None
    return C.c_void_p(t.data_ptr())


def _stream(s):
    if s is None:
        return None
    return C.c_void_p(s.cuda_stream)


_DT = {"f32": RTP_F32, "bf16": RTP_BF16, "f16": RTP_F16}


class Ring:
    """rtp_ring with its caller-owned buffers kept alive."""

    def __init__(self, n, rank, mode, w_bytes, g_bytes, home_w=None, home_g=None, buf_w=(None, None),
                 buf_g=(None, None), compute_stream=None, stage_stream=None, flags=0, aux_stream=None):
        d = rtp_ring_desc()
        d.n, d.rank, d.mode, d.flags = n, rank, mode, flags
        d.w_bytes, d.g_bytes = w_bytes, g_bytes
        d.home_w_dev, d.home_g_dev = _ptr(home_w), _ptr(home_g)
        d.buf_w_dev[0], d.buf_w_dev[1] = _ptr(buf_w[0]), _ptr(buf_w[1])
        d.buf_g_dev[0], d.buf_g_dev[1] = _ptr(buf_g[0]), _ptr(buf_g[1])
        d.compute_stream, d.stage_stream = _stream(compute_stream), _stream(stage_stream)
        d.aux_stream = _stream(aux_stream)
        self._keep = (home_w, home_g, buf_w, buf_g, compute_stream, stage_stream, aux_stream)
        self.desc = d
        self.handle = C.c_void_p()
        check(lib.rtp_ring_create(C.byref(self.handle), C.byref(d)), "rtp_ring_create")
        self.linears = []

    def begin(self, pass_):
        check(lib.rtp_ring_begin(self.handle, pass_), "rtp_ring_begin")

    def seek_bwd_start(self):
        check(lib.rtp_ring_seek_bwd_start(self.handle), "rtp_ring_seek_bwd_start")

    def rotate_step(self, direction, step):
        check(lib.rtp_rotate_step(self.handle, direction, step), "rtp_rotate_step")

    def end(self):
        check(lib.rtp_ring_end(self.handle), "rtp_ring_end")

    def abort(self):
        check(lib.rtp_ring_abort(self.handle), "rtp_ring_abort")

    def set_ablation(self, rotate=True, compute=True):
        check(lib.rtp_ring_set_ablation(self.handle, int(rotate), int(compute)), "rtp_ring_set_ablation")

    def flush(self):
        check(lib.rtp_ring_flush(self.handle), "rtp_ring_flush")

    def zero_grads(self):
        check(lib.rtp_ring_zero_grads(self.handle), "rtp_ring_zero_grads")

    def sync(self):
        check(lib.rtp_ring_sync(self.handle), "rtp_ring_sync")

    def resident(self):
        return lib.rtp_ring_resident(self.handle)

    def resident_grad(self):
        return lib.rtp_ring_resident_grad(self.handle)

    def trace(self, clear=False):
        total = lib.rtp_ring_trace(self.handle, None, 0, 0)
        buf = (rtp_trace_rec * max(total, 1))()
        lib.rtp_ring_trace(self.handle, buf, total, int(clear))
        return [(TRACE_KINDS[r.kind], r.pass_, r.step, r.shard, r.buffer) for r in buf[:total]]

    def close(self):
        for l in list(self.linears):
            l.close()
        if self.handle:
            check(lib.rtp_ring_destroy(self.handle), "rtp_ring_destroy")
            self.handle = C.c_void_p()


class Linear:
    def __init__(self, ring, T, I, O, split, dtype, act=RTP_ACT_NONE, w_offset=0, g_offset=0, preact=None,
                 acc_ws=None, grad_dtype=RTP_F32, has_bias=False):
        d = rtp_linear_desc()
        d.T, d.I, d.O = T, I, O
        d.split, d.dtype, d.grad_dtype, d.act = split, dtype, grad_dtype, act
        d.w_offset, d.g_offset = w_offset, g_offset
        d.preact_dev, d.acc_ws_dev = _ptr(preact), _ptr(acc_ws)
        d.has_bias = int(bool(has_bias))
        self._keep = (preact, acc_ws)
        self.ring = ring
        self.handle = C.c_void_p()
        check(lib.rtp_linear_create(C.byref(self.handle), ring.handle, C.byref(d)), "rtp_linear_create")
        ring.linears.append(self)

    def fwd(self, step, X, Y):
        check(lib.rtp_linear_fwd(self.handle, step, _ptr(X), _ptr(Y)), "rtp_linear_fwd")

    def bwd(self, step, X, dY, dX):
        check(lib.rtp_linear_bwd(self.handle, step, _ptr(X), _ptr(dY), _ptr(dX)), "rtp_linear_bwd")

    def fwd_noalloc(self, step, X, Y):
        check(lib.rtp_linear_fwd_noalloc(self.handle, step, _ptr(X), _ptr(Y)), "rtp_linear_fwd_noalloc")

    def close(self):
        if self.handle:
            check(lib.rtp_linear_destroy(self.handle), "rtp_linear_destroy")
            self.handle = C.c_void_p()
            self.ring.linears.remove(self)


def rtp_pack_shards(home, slot_bytes, offset, n, split, W, O, I, width, dtype, stream=None):
    """W[O, I] -> the n slots of `home` (a tensor or a raw device address), shard k's part at k * slot_bytes + offset."""
    hp = home if isinstance(home, (int, C.c_void_p)) else _ptr(home)
    check(lib.rtp_pack_shards(hp, slot_bytes, offset, n, split, _ptr(W), O, I, width, dtype, _stream(stream)), "rtp_pack_shards")


def rtp_unpack_shards(W, home, slot_bytes, offset, n, split, O, I, width, dtype, stream=None):
    hp = home if isinstance(home, (int, C.c_void_p)) else _ptr(home)
    check(lib.rtp_unpack_shards(_ptr(W), hp, slot_bytes, offset, n, split, O, I, width, dtype, _stream(stream)), "rtp_unpack_shards")


def rtp_gemm(layout, in_dtype, out_dtype, accumulate, A, lda, B, ldb, Cmat, ldc, M, N, K, variant=0, stream=None):
    check(lib.rtp_gemm(layout, in_dtype, out_dtype, int(accumulate), _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat), ldc,
                       M, N, K, variant, _stream(stream)), "rtp_gemm")


def rtp_gemm_kernel_name(layout, variant):
    return lib.rtp_gemm_kernel_name(layout, variant).decode()


def rtp_prof_begin(alone=False):
    check(lib.rtp_prof_begin_alone(int(alone)), "rtp_prof_begin")


def rtp_prof_end():
    """{layout name: (launches, total_ms, total_flops)}"""
    out = (rtp_prof_result * 3)()
    check(lib.rtp_prof_end(out), "rtp_prof_end")
    return {name: (out[i].launches, out[i].total_ms, out[i].total_flops) for i, name in enumerate(("nt", "nn", "tn"))}


def rtp_clock_probe(stream, out, wall_us):
    """Enqueue the clock probe on `stream`; `out` is an int64[2] device tensor.  Returns the wall
    clock's rate in kHz; after the stream has drained, out[1] / out[0] * kHz is the shader clock."""
    khz = C.c_int(0)
    check(lib.rtp_clock_probe(_stream(stream), _ptr(out), int(wall_us), C.byref(khz)), "rtp_clock_probe")
    return khz.value
