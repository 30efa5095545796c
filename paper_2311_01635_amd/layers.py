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
    streams into the compute stream)."""

    def _enter(self):
        self.compute_stream.wait_stream(torch.cuda.current_stream(self.dev))

    def _leave(self):
        torch.cuda.current_stream(self.dev).wait_stream(self.compute_stream)


def pack_out_split(W, n, o=None):
    """[O, I] -> [n, o*I]: shard k is rows [k o, (k+1) o); rows past O (padded partition) are zero."""
    O, I = W.shape
    o = O // n if o is None else o
    if n * o != O:
        W = torch.cat((W, W.new_zeros(n * o - O, I)), dim=0)
    return W.reshape(n, o * I).clone()       # a store of its own: the ring writes into it


def pack_in_split(W, n, o=None):
    """[O, I] -> [n, O*o]: shard k is columns [k o, (k+1) o), stored [O, o]; columns past I are zero."""
    O, I = W.shape
    o = I // n if o is None else o
    if n * o != I:
        W = torch.cat((W, W.new_zeros(O, n * o - I)), dim=1)
    return W.reshape(O, n, o).permute(1, 0, 2).clone(memory_format=torch.contiguous_format).reshape(n, O * o)


def unpack_out_split(P, n, O, I):
    return P.reshape(-1, I)[:O].contiguous()


def unpack_in_split(P, n, O, I):
    o = P.shape[1] // O
    return P.reshape(n, O, o).permute(1, 0, 2).reshape(O, n * o)[:, :I].contiguous()


def stack_gate_up(Wg, Wu, n):
    """[O, I] x 2 -> [2 O, I] with shard k = gate rows k followed by up rows k."""
    O, I = Wg.shape
    o = O // n
    return torch.stack((Wg.reshape(n, o, I), Wu.reshape(n, o, I)), dim=1).reshape(2 * O, I).contiguous()


def unstack_gate_up(Wgu, n):
    O2, I = Wgu.shape
    o = O2 // (2 * n)
    v = Wgu.reshape(n, 2, o, I)
    return v[:, 0].reshape(n * o, I).contiguous(), v[:, 1].reshape(n * o, I).contiguous()


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
        pack = pack_out_split if split == B.RTP_SPLIT_OUT else pack_in_split
        o = B.lib.rtp_shard_width(self.O if split == B.RTP_SPLIT_OUT else self.I, n, dtype)
        if o <= 0:
            raise ValueError("the partitioned dimension cannot be split into n non-empty aligned shards")
        self.o, self.has_bias = o, bias is not None
        self.home_w = pack(W, n, o).contiguous()
        G0 = torch.zeros(self.O, self.I, device=self.dev, dtype=torch.float32) if G0 is None else \
            G0.to(self.dev, torch.float32)
        self.home_g = pack(G0, n, o).contiguous()
        self.n_mat = self.home_w.shape[1]                  # elements of a matrix shard
        if self.has_bias:
            # shard k of the flat parameter = its rows of W, then its entries of b, padded to 16 bytes
            d = B.rtp_linear_desc()
            d.T, d.I, d.O, d.split, d.dtype, d.grad_dtype, d.has_bias = T, self.I, self.O, split, dtype, B.RTP_F32, 1
            wbytes, gbytes = B.lib.rtp_linear_shard_w_bytes(C.byref(d), n), B.lib.rtp_linear_shard_g_bytes(C.byref(d), n)
            # (an input-partitioned layer spreads b over the shards in pieces of rtp_bias_piece_width entries)
            pw = self.pw = o if split == B.RTP_SPLIT_OUT else B.lib.rtp_bias_piece_width(self.O, n, dtype)

            def with_bias(mat, vec, total):
                vec = torch.cat((vec, vec.new_zeros(n * pw - vec.numel()))).reshape(n, pw)
                out = mat.new_zeros(n, total)
                out[:, :self.n_mat] = mat
                out[:, self.n_mat:self.n_mat + pw] = vec
                return out.contiguous()
            gb0 = torch.zeros(self.O, device=self.dev) if gb0 is None else gb0
            self.home_w = with_bias(self.home_w, bias.to(self.dev, td), wbytes // _esize(dtype))
            self.home_g = with_bias(self.home_g, gb0.to(self.dev, torch.float32), gbytes // 4)
        wb = self.home_w.shape[1] * _esize(dtype)
        gb = self.home_g.shape[1] * 4
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

    def zero_grads(self):
        self.ring.zero_grads()

    def gathered(self):
        """(W, G) as full matrices, read back from the home store."""
        self.ring.flush()
        self.ring.sync()
        un = unpack_out_split if self.split == B.RTP_SPLIT_OUT else unpack_in_split
        return (un(self.home_w[:, :self.n_mat].contiguous(), self.n, self.O, self.I),
                un(self.home_g[:, :self.n_mat].contiguous(), self.n, self.O, self.I))

    def gathered_bias(self):
        """(b, gradient of b) read back from the home store (call gathered() first: it flushes)."""
        sl = slice(self.n_mat, self.n_mat + self.pw)
        return self.home_w[:, sl].reshape(-1)[:self.O].contiguous(), self.home_g[:, sl].reshape(-1)[:self.O].contiguous()

    def close(self):
        self.ring.close()


class RtpMlp(_PassStreams):
    """MLP unit (first GEMM output-partitioned, second input-partitioned) run
    by rtp_mlp_fwd / rtp_mlp_bwd: one library call per pass."""

    def __init__(self, weights, T, n, rank, act, mode=B.RTP_INPLACE_STAGED, dtype=B.RTP_BF16, G0=None,
                 device="cuda:0", aux_stream=True, stepwise=False, biases=None, gb0=None, grouped=False, pipelined=False, stage_memcpy=False):
        self.dev = torch.device(device)
        td = _TORCH_DT[dtype]
        self.n, self.rank, self.T, self.act, self.mode, self.dtype = n, rank, T, act, mode, dtype
        self.gated = act == B.RTP_ACT_SWIGLU
        self.has_bias = biases is not None
        ws = [w.to(self.dev, td).contiguous() for w in weights]
        if self.gated:
            Wg, Wu, Wd = ws
            W1 = stack_gate_up(Wg, Wu, n)
        else:
            W1, Wd = ws
        self.O, self.I = (W1.shape[0] // 2 if self.gated else W1.shape[0]), W1.shape[1]
        self.O2 = Wd.shape[0]
        self.p = 2 if self.gated else 1
        self.n1 = self.p * self.O * self.I // n           # elements of the first matrix's shard
        self.n2 = self.O2 * self.O // n
        d = B.rtp_mlp_desc()
        d.T, d.I, d.O, d.O2 = T, self.I, self.O, self.O2
        d.n, d.rank, d.mode, d.dtype, d.act = n, rank, mode, dtype, act
        d.flags = ((B.RTP_FLAG_STEPWISE if stepwise else 0) | (B.RTP_FLAG_GROUPED if grouped else 0) |
                   (B.RTP_FLAG_PIPELINED if pipelined else 0) | (B.RTP_FLAG_STAGE_MEMCPY if stage_memcpy else 0))
        d.has_bias = int(self.has_bias)
        wb, gb = B.lib.rtp_mlp_slot_w_bytes(C.byref(d)), B.lib.rtp_mlp_slot_g_bytes(C.byref(d))
        g = None if G0 is None else [x.to(self.dev, torch.float32) for x in G0]
        G1 = None if g is None else (stack_gate_up(g[0], g[1], n) if self.gated else g[0])
        if not self.has_bias:
            self.off2 = self.n1                           # where the second linear's part starts, in elements
            self.home_w = torch.cat((pack_out_split(W1, n), pack_in_split(Wd, n)), dim=1).contiguous()
            if G0 is None:
                self.home_g = torch.zeros(n, self.n1 + self.n2, dtype=torch.float32, device=self.dev)
            else:
                self.home_g = torch.cat((pack_out_split(G1, n), pack_in_split(g[-1], n)), dim=1).contiguous()
        else:
            # slot = [W1_k | b1_k | W2_k | piece k of b2]; each linear's part is padded to 16 bytes in the
            # weight type and in fp32 alike, so one element offset serves both stores
            self.o1 = self.O // n
            self.pw2 = B.lib.rtp_bias_piece_width(self.O2, n, dtype)
            l1 = B.rtp_linear_desc()
            l1.T, l1.I, l1.O, l1.split, l1.dtype, l1.grad_dtype, l1.has_bias = T, self.I, self.O, B.RTP_SPLIT_OUT, dtype, B.RTP_F32, 1
            self.off2 = B.lib.rtp_linear_shard_w_bytes(C.byref(l1), n) // _esize(dtype)
            assert self.off2 * 4 == B.lib.rtp_linear_shard_g_bytes(C.byref(l1), n)
            gb0 = [torch.zeros(self.O), torch.zeros(self.O2)] if gb0 is None else gb0

            def slot(M1, v1, M2, v2, t, total):
                out = torch.zeros(n, total, dtype=t, device=self.dev)
                out[:, :self.n1] = pack_out_split(M1.to(self.dev, t), n)
                out[:, self.n1:self.n1 + self.o1] = v1.to(self.dev, t).reshape(n, self.o1)
                out[:, self.off2:self.off2 + self.n2] = pack_in_split(M2.to(self.dev, t), n)
                v2 = v2.to(self.dev, t)
                v2 = torch.cat((v2, v2.new_zeros(n * self.pw2 - v2.numel()))).reshape(n, self.pw2)
                out[:, self.off2 + self.n2:self.off2 + self.n2 + self.pw2] = v2
                return out.contiguous()

            self.home_w = slot(W1, biases[0], Wd, biases[1], td, wb // _esize(dtype))
            Z1, Z2 = torch.zeros(self.O, self.I), torch.zeros(self.O2, self.O)
            self.home_g = slot(Z1 if g is None else G1, gb0[0], Z2 if g is None else g[-1], gb0[1], torch.float32, gb // 4)
        assert wb == self.home_w.shape[1] * _esize(dtype) and gb == self.home_g.shape[1] * 4
        self.w_bytes, self.g_bytes = wb, gb
        self.buf_w = [torch.empty(wb, dtype=torch.uint8, device=self.dev) for _ in range(2)]
        ng = 2 if mode == B.RTP_DOUBLE_BUFFER else 1
        self.buf_g = [torch.empty(gb, dtype=torch.uint8, device=self.dev) for _ in range(ng)] + [None] * (2 - ng)
        self.preact = torch.empty(T, self.p * self.O, dtype=td, device=self.dev)
        self.hidden = torch.empty(T, self.O, dtype=td, device=self.dev)
        self.dpre = torch.empty(T, self.p * self.O, dtype=td, device=self.dev)
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
        out = []
        for home in (self.home_w, self.home_g):
            P1, P2 = home[:, :self.n1].contiguous(), home[:, self.off2:self.off2 + self.n2].contiguous()
            M1 = unpack_out_split(P1, self.n, self.p * self.O, self.I)
            M2 = unpack_in_split(P2, self.n, self.O2, self.O)
            out.append((*unstack_gate_up(M1, self.n), M2) if self.gated else (M1, M2))
        return out

    def gathered_biases(self):
        """((b1, b2), (gradient of b1, gradient of b2)) from the home store (call gathered() first: it flushes)."""
        out = []
        for home in (self.home_w, self.home_g):
            v1 = home[:, self.n1:self.n1 + self.o1].reshape(-1).contiguous()
            s2 = self.off2 + self.n2
            v2 = home[:, s2:s2 + self.pw2].reshape(-1)[:self.O2].contiguous()
            out.append((v1, v2))
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

        def slot(mats, t):
            # [W1_e | W2_e], W1_e = [gate_e ; up_e] for a gated expert: every matrix flattened row-major
            return torch.cat([m.to(self.dev, t).contiguous().reshape(-1) for m in mats])

        self.home_w = torch.stack([slot(ex, td) for ex in experts]).contiguous()
        if G0 is None:
            self.home_g = torch.zeros(n, self.home_w.shape[1], dtype=torch.float32, device=self.dev)
        else:
            self.home_g = torch.stack([slot(g, torch.float32) for g in G0]).contiguous()
        d = B.rtp_moe_desc()
        d.T, d.I, d.O, d.O2 = T, self.I, self.O, self.O2
        d.n, d.rank, d.mode, d.dtype, d.act, d.flags = n, rank, mode, dtype, act, 0
        wb, gb = B.lib.rtp_moe_slot_w_bytes(C.byref(d)), B.lib.rtp_moe_slot_g_bytes(C.byref(d))
        assert wb == self.home_w.shape[1] * _esize(dtype) and gb == self.home_g.shape[1] * 4
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
        for home in (self.home_w, self.home_g):
            per = []
            for e in range(self.n):
                mats, off = [], 0
                for (r, c) in self.shapes:
                    mats.append(home[e, off:off + r * c].reshape(r, c).clone())
                    off += r * c
                per.append(tuple(mats))
            out.append(per)
        return out

    def close(self):
        if self.handle:
            B.check(B.lib.rtp_moe_destroy(self.handle), "rtp_moe_destroy")
            self.handle = C.c_void_p()
