"""Torch-side plumbing: device buffers, streams and the packing of full
matrices into the ring store.  No arithmetic of the method happens here; the
forward and backward steps are calls into librtp.so."""
import ctypes as C

import torch

from . import binding as B

_TORCH_DT = {B.RTP_F32: torch.float32, B.RTP_BF16: torch.bfloat16, B.RTP_F16: torch.float16}


def _esize(dtype):
    return 4 if dtype == B.RTP_F32 else 2


class _PassStreams:
    """Orders a layer's private streams with the caller's: a pass starts after everything the
    caller's current stream holds (X, dY or the routing may just have been produced there) and the
    caller's stream continues after the pass (rtp_ring_end has joined the stage and auxiliary
    streams into the compute stream).  A caller whose current stream IS the layer's compute stream
    (`with torch.cuda.stream(layer.compute_stream):`) skips both hops."""

    def _enter(self):
        cur = torch.cuda.current_stream(self.dev)
        if cur != self.compute_stream:        # a caller that runs on the layer's compute stream needs no hop
            self.compute_stream.wait_stream(cur)

    def _leave(self):
        cur = torch.cuda.current_stream(self.dev)
        if cur != self.compute_stream:
            cur.wait_stream(self.compute_stream)


class _Store:
    """The ring store of one unit: `n` slots of `slot_bytes` each (a uint8 tensor), written and read through
    rtp_pack_shards / rtp_unpack_shards.  `parts` remembers where each full matrix (or bias vector) lives."""

    def __init__(self, n, slot_bytes, dtype, device):
        self.n, self.slot_bytes, self.dtype = n, slot_bytes, dtype
        self.es = _esize(dtype)
        self.buf = torch.zeros(n, slot_bytes, dtype=torch.uint8, device=device)   # padding between parts stays zero
        self.parts = {}

    def pack(self, name, M, offset, split, width):
        """Matrix M [O, I] (a vector counts as [O, 1]) into the store at `offset` bytes of every slot."""
        M2 = M.reshape(M.shape[0], -1).to(self.buf.device, _TORCH_DT[self.dtype]).contiguous()
        O, I = M2.shape
        self.parts[name] = (offset, split, O, I, width, tuple(M.shape))
        B.rtp_pack_shards(self.buf, self.slot_bytes, offset, self.n, split, M2, O, I, width, self.dtype)

    def unpack(self, name):
        offset, split, O, I, width, shape = self.parts[name]
        out = torch.empty(O, I, dtype=_TORCH_DT[self.dtype], device=self.buf.device)
        B.rtp_unpack_shards(out, self.buf, self.slot_bytes, offset, self.n, split, O, I, width, self.dtype)
        return out.reshape(shape)


class RtpLinear(_PassStreams):
    """One rotated linear layer: the N-step loop issued call by call through
    rtp_rotate_step / rtp_linear_fwd / rtp_linear_bwd."""

    def __init__(self, W, T, n, rank, split=B.RTP_SPLIT_OUT, mode=B.RTP_DOUBLE_BUFFER, dtype=B.RTP_BF16,
                 act=B.RTP_ACT_NONE, G0=None, preact=None, device="cuda:0", aux_stream=True, bias=None, gb0=None):
        self.dev = torch.device(device)
        self.n, self.rank, self.T, self.split, self.mode, self.dtype, self.act = n, rank, T, split, mode, dtype, act
        td = _TORCH_DT[dtype]
        W = W.to(self.dev, td).contiguous()
        self.O, self.I = W.shape
        o = B.lib.rtp_shard_width(self.O if split == B.RTP_SPLIT_OUT else self.I, n, dtype)
        if o <= 0:
            raise ValueError("the partitioned dimension cannot be split into n non-empty aligned shards")
        self.o, self.has_bias = o, bias is not None
        d = B.rtp_linear_desc()
        d.T, d.I, d.O, d.split, d.dtype, d.grad_dtype, d.has_bias = T, self.I, self.O, split, dtype, B.RTP_F32, int(self.has_bias)
        wb, gb = B.lib.rtp_linear_shard_w_bytes(C.byref(d), n), B.lib.rtp_linear_shard_g_bytes(C.byref(d), n)
        # the shard layout is the library's (rtp_pack_shards): shard k of the flat parameter = its block of W,
        # then (with a bias) its entries of b -- for an input-partitioned layer piece k of b
        self.store_w, self.store_g = _Store(n, wb, dtype, self.dev), _Store(n, gb, B.RTP_F32, self.dev)
        G0 = torch.zeros(self.O, self.I, device=self.dev, dtype=torch.float32) if G0 is None else G0
        self.store_w.pack("W", W, 0, split, o)
        self.store_g.pack("W", G0, 0, split, o)
        n_mat = o * (self.I if split == B.RTP_SPLIT_OUT else self.O)      # elements of a matrix shard
        if self.has_bias:
            pw = o if split == B.RTP_SPLIT_OUT else B.lib.rtp_bias_piece_width(self.O, n, dtype)
            gb0 = torch.zeros(self.O, device=self.dev) if gb0 is None else gb0
            self.store_w.pack("b", bias, n_mat * _esize(dtype), B.RTP_SPLIT_OUT, pw)
            self.store_g.pack("b", gb0, n_mat * 4, B.RTP_SPLIT_OUT, pw)
        self.home_w, self.home_g = self.store_w.buf, self.store_g.buf
        self.buf_w = [torch.empty(wb, dtype=torch.uint8, device=self.dev) for _ in range(2)]
        self.buf_g = [torch.empty(gb, dtype=torch.uint8, device=self.dev) for _ in range(2)]
        self.compute_stream = torch.cuda.Stream(self.dev)
        self.stage_stream = torch.cuda.Stream(self.dev)
        self.aux_stream = torch.cuda.Stream(self.dev) if aux_stream else None
        self.ring = B.Ring(n, rank, mode, wb, gb, self.home_w, self.home_g, self.buf_w, self.buf_g,
                           self.compute_stream, self.stage_stream, aux_stream=self.aux_stream)
        acc_cols = self.I if split == B.RTP_SPLIT_OUT else self.O
        self.acc_ws = torch.empty(T, acc_cols, dtype=torch.float32, device=self.dev)
        self.preact = preact
        self.lin = B.Linear(self.ring, T, self.I, self.O, split, dtype, act, 0, 0, preact, self.acc_ws,
                            has_bias=self.has_bias)
        torch.cuda.synchronize(self.dev)

    def forward(self, X, Y):
        r, n = self.ring, self.n
        self._enter()
        r.begin(B.RTP_PASS_FWD)
        for t in range(n):
            if t < n - 1:
                r.rotate_step(B.RTP_CW, t)
            self.lin.fwd(t, X, Y)
        r.end()
        self._leave()

    def backward(self, X, dY, dX):
        r, n = self.ring, self.n
        self._enter()
        r.begin(B.RTP_PASS_BWD)
        for s in range(n):
            if s < n - 1:
                r.rotate_step(B.RTP_CCW, s)
            self.lin.bwd(s, X, dY, dX)
        r.end()
        self._leave()

    def sync(self):
        self.ring.sync()

    def set_ablation(self, rotate=True, compute=True):
        self.ring.set_ablation(rotate, compute)

    def worker_bytes(self):
        return B.rtp_worker_bytes(self.mode, self.ring.desc.w_bytes, self.ring.desc.g_bytes)

    def zero_grads(self):
        self.ring.zero_grads()

    def gathered(self):
        """(W, G) as full matrices, read back from the home store."""
        self.ring.flush()
        self.ring.sync()
        out = self.store_w.unpack("W"), self.store_g.unpack("W")
        torch.cuda.synchronize(self.dev)
        return out

    def gathered_bias(self):
        """(b, gradient of b) read back from the home store (call gathered() first: it flushes)."""
        out = self.store_w.unpack("b"), self.store_g.unpack("b")
        torch.cuda.synchronize(self.dev)
        return out

    def close(self):
        self.ring.close()


class RtpMlp(_PassStreams):
    """MLP unit (first GEMM output-partitioned, second input-partitioned) run
    by rtp_mlp_fwd / rtp_mlp_bwd: one library call per pass."""

    def __init__(self, weights, T, n, rank, act, mode=B.RTP_INPLACE_STAGED, dtype=B.RTP_BF16, G0=None,
                 device="cuda:0", aux_stream=True, stepwise=False, biases=None, gb0=None, grouped=False, pipelined=False, stage_memcpy=False, fused=False):
        self.dev = torch.device(device)
        td = _TORCH_DT[dtype]
        self.n, self.rank, self.T, self.act, self.mode, self.dtype = n, rank, T, act, mode, dtype
        self.gated = act == B.RTP_ACT_SWIGLU
        self.has_bias = biases is not None
        ws = [w.to(self.dev, td).contiguous() for w in weights]
        self.names = ("Wg", "Wu", "Wd") if self.gated else ("W1", "W2")
        self.O, self.I = ws[0].shape
        self.O2 = ws[-1].shape[0]
        self.p = 2 if self.gated else 1
        d = B.rtp_mlp_desc()
        d.T, d.I, d.O, d.O2 = T, self.I, self.O, self.O2
        d.n, d.rank, d.mode, d.dtype, d.act = n, rank, mode, dtype, act
        d.flags = ((B.RTP_FLAG_STEPWISE if stepwise else 0) | (B.RTP_FLAG_GROUPED if grouped else 0) |
                   (B.RTP_FLAG_PIPELINED if pipelined else 0) | (B.RTP_FLAG_STAGE_MEMCPY if stage_memcpy else 0) |
                   (B.RTP_FLAG_FUSED_STEP if fused else 0))
        d.has_bias = int(self.has_bias)
        wb, gb = B.lib.rtp_mlp_slot_w_bytes(C.byref(d)), B.lib.rtp_mlp_slot_g_bytes(C.byref(d))
        if wb == 0 or gb == 0:
            raise ValueError("rtp_mlp_slot_*_bytes rejects this unit (sizes, or a partition the unit does not take)")
        self.w_bytes, self.g_bytes = wb, gb
        # Slot k = [first linear's shard | second linear's shard]; the first linear's shard is its row block of W1
        # (gated unit: gate rows k, then up rows k), then its bias entries; the second's is its column block of
        # W2 stored [O2, o], then piece k of its bias.  Offsets are the library's (rtp_linear_shard_*_bytes); the
        # layout itself is written by rtp_pack_shards.  Gradient store: the same, fp32.
        hw = self.hidden_width = B.lib.rtp_mlp_hidden_width(C.byref(d))   # O, or n shards of the padded width
        o = hw // n                                          # hidden units per shard
        l1 = B.rtp_linear_desc()
        l1.T, l1.I, l1.O, l1.split, l1.dtype, l1.grad_dtype = T, self.I, self.p * hw, B.RTP_SPLIT_OUT, dtype, B.RTP_F32
        l1.act, l1.has_bias = act, int(self.has_bias)
        off2_w, off2_g = B.lib.rtp_linear_shard_w_bytes(C.byref(l1), n), B.lib.rtp_linear_shard_g_bytes(C.byref(l1), n)
        assert off2_w // _esize(dtype) == off2_g // 4
        self.store_w, self.store_g = _Store(n, wb, dtype, self.dev), _Store(n, gb, B.RTP_F32, self.dev)
        zeros = lambda *shape: torch.zeros(*shape, dtype=torch.float32, device=self.dev)
        g = [zeros(*w.shape) for w in ws] if G0 is None else list(G0)
        bs = list(biases) if self.has_bias else []
        gbs = ([zeros(b.numel()) for b in bs] if gb0 is None else list(gb0)) if self.has_bias else []
        for store, mats, vecs, es, off2 in ((self.store_w, ws, bs, _esize(dtype), off2_w), (self.store_g, g, gbs, 4, off2_g)):
            for j in range(self.p):                           # W1, or gate then up: o rows of I each
                store.pack(self.names[j], mats[j], j * o * self.I * es, B.RTP_SPLIT_OUT, o)
            store.pack(self.names[-1], mats[-1], off2, B.RTP_SPLIT_IN, o)
            if self.has_bias:
                for j in range(self.p):                       # the first linear's bias entries follow its rows
                    store.pack("b" + self.names[j], vecs[j], (self.p * o * self.I + j * o) * es, B.RTP_SPLIT_OUT, o)
                pw2 = B.lib.rtp_bias_piece_width(self.O2, n, dtype)
                store.pack("b" + self.names[-1], vecs[-1], off2 + self.O2 * o * es, B.RTP_SPLIT_OUT, pw2)
        self.home_w, self.home_g = self.store_w.buf, self.store_g.buf
        self.buf_w = [torch.empty(wb, dtype=torch.uint8, device=self.dev) for _ in range(2)]
        ng = 2 if mode == B.RTP_DOUBLE_BUFFER else 1
        self.buf_g = [torch.empty(gb, dtype=torch.uint8, device=self.dev) for _ in range(ng)] + [None] * (2 - ng)
        self.preact = torch.empty(T, self.p * hw, dtype=td, device=self.dev)
        self.hidden = torch.empty(T, hw, dtype=td, device=self.dev)
        self.dpre = torch.empty(T, self.p * hw, dtype=td, device=self.dev)
        self.acc_y = torch.empty(T, self.O2, dtype=torch.float32, device=self.dev)
        self.acc_dx = torch.empty(T, self.I, dtype=torch.float32, device=self.dev)
        self.compute_stream = torch.cuda.Stream(self.dev)
        self.stage_stream = torch.cuda.Stream(self.dev)
        d.home_w_dev, d.home_g_dev = B._ptr(self.home_w), B._ptr(self.home_g)
        d.buf_w_dev[0], d.buf_w_dev[1] = B._ptr(self.buf_w[0]), B._ptr(self.buf_w[1])
        d.buf_g_dev[0], d.buf_g_dev[1] = B._ptr(self.buf_g[0]), B._ptr(self.buf_g[1])
        d.preact_dev, d.hidden_dev, d.dpre_dev = B._ptr(self.preact), B._ptr(self.hidden), B._ptr(self.dpre)
        d.acc_y_dev, d.acc_dx_dev = B._ptr(self.acc_y), B._ptr(self.acc_dx)
        d.compute_stream, d.stage_stream = B._stream(self.compute_stream), B._stream(self.stage_stream)
        self.aux_stream = torch.cuda.Stream(self.dev) if aux_stream else None
        d.aux_stream = B._stream(self.aux_stream)
        self.step_sync = torch.zeros(B.lib.rtp_mlp_step_sync_bytes(C.byref(d)), dtype=torch.uint8, device=self.dev) if fused else None
        d.step_sync_dev = B._ptr(self.step_sync)
        self.desc = d
        self.handle = C.c_void_p()
        B.check(B.lib.rtp_mlp_create(C.byref(self.handle), C.byref(d)), "rtp_mlp_create")
        torch.cuda.synchronize(self.dev)

    def forward(self, X, Y):
        self._enter()
        B.check(B.lib.rtp_mlp_fwd(self.handle, B._ptr(X), B._ptr(Y)), "rtp_mlp_fwd")
        self._leave()

    def backward(self, X, dY, dX):
        self._enter()
        B.check(B.lib.rtp_mlp_bwd(self.handle, B._ptr(X), B._ptr(dY), B._ptr(dX)), "rtp_mlp_bwd")
        self._leave()

    def set_ablation(self, rotate=True, compute=True):
        B.check(B.lib.rtp_mlp_set_ablation(self.handle, int(rotate), int(compute)), "rtp_mlp_set_ablation")

    def sync(self):
        B.check(B.lib.rtp_mlp_sync(self.handle), "rtp_mlp_sync")

    def zero_grads(self):
        B.check(B.lib.rtp_ring_zero_grads(B.lib.rtp_mlp_ring(self.handle)), "rtp_ring_zero_grads")

    def worker_bytes(self):
        return B.rtp_worker_bytes(self.mode, self.w_bytes, self.g_bytes)

    def gathered(self):
        """Full matrices read back from the home store: (weights, gradients)
        in the order they were given."""
        B.check(B.lib.rtp_mlp_flush(self.handle), "rtp_mlp_flush")
        self.sync()
        out = [tuple(store.unpack(nm) for nm in self.names) for store in (self.store_w, self.store_g)]
        torch.cuda.synchronize(self.dev)
        return out

    def gathered_biases(self):
        """(biases, their gradients), each in the order the matrices were given, from the home store (call
        gathered() first: it flushes)."""
        out = [tuple(store.unpack("b" + nm) for nm in self.names) for store in (self.store_w, self.store_g)]
        torch.cuda.synchronize(self.dev)
        return out

    def close(self):
        if self.handle:
            B.check(B.lib.rtp_mlp_destroy(self.handle), "rtp_mlp_destroy")
            self.handle = C.c_void_p()


class RtpMoe(_PassStreams):
    """Expert-partitioned layer run by rtp_moe_fwd / rtp_moe_bwd: the ring's
    shard is one whole expert.  `experts[e]` = (W1, W2) or (Wg, Wu, Wd)."""

    def __init__(self, experts, T, rank, act, mode=B.RTP_INPLACE_STAGED, dtype=B.RTP_BF16, G0=None,
                 device="cuda:0", aux_stream=True):
        self.dev = torch.device(device)
        td = _TORCH_DT[dtype]
        n = len(experts)
        self.n, self.rank, self.T, self.act, self.mode, self.dtype = n, rank, T, act, mode, dtype
        self.gated = act == B.RTP_ACT_SWIGLU
        self.shapes = [tuple(w.shape) for w in experts[0]]
        self.O, self.I = self.shapes[0]
        self.O2 = self.shapes[-1][0]
        self.p = 2 if self.gated else 1

        d = B.rtp_moe_desc()
        d.T, d.I, d.O, d.O2 = T, self.I, self.O, self.O2
        d.n, d.rank, d.mode, d.dtype, d.act, d.flags = n, rank, mode, dtype, act, 0
        wb, gb = B.lib.rtp_moe_slot_w_bytes(C.byref(d)), B.lib.rtp_moe_slot_g_bytes(C.byref(d))
        # slot e = [W1_e | W2_e] (W1_e = [gate_e ; up_e] for a gated expert), every matrix whole and row-major:
        # one rtp_pack_shards call per matrix with n = 1, aimed at the expert's slot
        self.home_w = torch.zeros(n, wb, dtype=torch.uint8, device=self.dev)
        self.home_g = torch.zeros(n, gb, dtype=torch.uint8, device=self.dev)
        self._offsets = []
        off = 0
        for (r, c) in self.shapes:
            self._offsets.append(off)
            off += r * c
        for e in range(n):
            for j, (r, c) in enumerate(self.shapes):
                B.rtp_pack_shards(self.home_w.data_ptr() + e * wb, wb, self._offsets[j] * _esize(dtype), 1, B.RTP_SPLIT_OUT,
                                  experts[e][j].to(self.dev, td).contiguous(), r, c, r, dtype)
                if G0 is not None:
                    B.rtp_pack_shards(self.home_g.data_ptr() + e * gb, gb, self._offsets[j] * 4, 1, B.RTP_SPLIT_OUT,
                                      G0[e][j].to(self.dev, torch.float32).contiguous(), r, c, r, B.RTP_F32)
        torch.cuda.synchronize(self.dev)
        self.w_bytes, self.g_bytes = wb, gb
        self.buf_w = [torch.empty(wb, dtype=torch.uint8, device=self.dev) for _ in range(2)]
        ng = 2 if mode == B.RTP_DOUBLE_BUFFER else 1
        self.buf_g = [torch.empty(gb, dtype=torch.uint8, device=self.dev) for _ in range(ng)] + [None] * (2 - ng)
        Tp = self.Tp = B.lib.rtp_moe_padded_rows(T, n)
        self.xp = torch.empty(Tp, self.I, dtype=td, device=self.dev)
        self.preact = torch.empty(Tp, self.p * self.O, dtype=td, device=self.dev)
        self.hidden = torch.empty(Tp, self.O, dtype=td, device=self.dev)
        self.yp = torch.empty(Tp, self.O2, dtype=td, device=self.dev)
        self.dpre = torch.empty(Tp, self.p * self.O, dtype=td, device=self.dev)
        self.dxp = torch.empty(Tp, self.I, dtype=td, device=self.dev)
        self.perm = torch.empty(Tp, dtype=torch.int32, device=self.dev)
        self.counts = torch.empty(n + 1, dtype=torch.int32, device=self.dev)
        self.compute_stream = torch.cuda.Stream(self.dev)
        self.stage_stream = torch.cuda.Stream(self.dev)
        self.aux_stream = torch.cuda.Stream(self.dev) if aux_stream else None
        d.home_w_dev, d.home_g_dev = B._ptr(self.home_w), B._ptr(self.home_g)
        d.buf_w_dev[0], d.buf_w_dev[1] = B._ptr(self.buf_w[0]), B._ptr(self.buf_w[1])
        d.buf_g_dev[0], d.buf_g_dev[1] = B._ptr(self.buf_g[0]), B._ptr(self.buf_g[1])
        d.xp_dev, d.preact_dev, d.hidden_dev = B._ptr(self.xp), B._ptr(self.preact), B._ptr(self.hidden)
        d.yp_dev, d.dpre_dev, d.dxp_dev = B._ptr(self.yp), B._ptr(self.dpre), B._ptr(self.dxp)
        d.perm_dev, d.counts_dev = B._ptr(self.perm), B._ptr(self.counts)
        d.compute_stream, d.stage_stream = B._stream(self.compute_stream), B._stream(self.stage_stream)
        d.aux_stream = B._stream(self.aux_stream) if aux_stream else None
        self.desc = d
        self.handle = C.c_void_p()
        torch.cuda.synchronize(self.dev)
        B.check(B.lib.rtp_moe_create(C.byref(self.handle), C.byref(d)), "rtp_moe_create")

    def forward(self, X, route, Y):
        self._enter()
        B.check(B.lib.rtp_moe_fwd(self.handle, B._ptr(X), B._ptr(route), B._ptr(Y)), "rtp_moe_fwd")
        self._leave()

    def backward(self, dY, dX):
        self._enter()
        B.check(B.lib.rtp_moe_bwd(self.handle, B._ptr(dY), B._ptr(dX)), "rtp_moe_bwd")
        self._leave()

    def sync(self):
        B.check(B.lib.rtp_moe_sync(self.handle), "rtp_moe_sync")

    def set_ablation(self, rotate=True, compute=True):
        B.check(B.lib.rtp_moe_set_ablation(self.handle, int(rotate), int(compute)), "rtp_moe_set_ablation")

    def worker_bytes(self):
        return B.rtp_worker_bytes(self.mode, self.w_bytes, self.g_bytes)

    def zero_grads(self):
        B.check(B.lib.rtp_ring_zero_grads(B.lib.rtp_moe_ring(self.handle)), "rtp_ring_zero_grads")

    def routing(self):
        """(tokens per expert, first grouped row of each expert) of the last forward."""
        c, b = (C.c_int32 * self.n)(), (C.c_int64 * (self.n + 1))()
        B.check(B.lib.rtp_moe_routing(self.handle, c, b), "rtp_moe_routing")
        return list(c), list(b)

    def gathered(self):
        """(weights, gradients), each a list over experts of the expert's matrices, from the home store."""
        B.check(B.lib.rtp_moe_flush(self.handle), "rtp_moe_flush")
        self.sync()
        out = []
        for home, slot, dt, es in ((self.home_w, self.w_bytes, self.dtype, _esize(self.dtype)), (self.home_g, self.g_bytes, B.RTP_F32, 4)):
            per = []
            for e in range(self.n):
                mats = []
                for j, (r, c) in enumerate(self.shapes):
                    m = torch.empty(r, c, dtype=_TORCH_DT[dt], device=self.dev)
                    B.rtp_unpack_shards(m, home.data_ptr() + e * slot, slot, self._offsets[j] * es, 1, B.RTP_SPLIT_OUT, r, c, r, dt)
                    mats.append(m)
                per.append(tuple(mats))
            out.append(per)
        torch.cuda.synchronize(self.dev)
        return out

    def close(self):
        if self.handle:
            B.check(B.lib.rtp_moe_destroy(self.handle), "rtp_moe_destroy")
            self.handle = C.c_void_p()
