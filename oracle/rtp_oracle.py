"""fp64 CPU oracle of the rotated-shard linear layer -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It shares nothing with the HIP library: the arithmetic lives in
rtp_oracle.c (triple loops, fp64) and this file only walks the rotation
schedule in the order the paper gives it, moving shards between a "home"
store (the other workers' memory), a resident buffer and a staging buffer
with explicit copies, so that the indexing can be checked, not just the sum.

Notation (Partition Strategies section): N workers ("partition factor"),
worker rank r, local tokens T, in-features I, out-features O, shard width
o = O/N.  W is stored [O, I] so that the forward is Y = X W^T; the paper
writes the same thing as GEMM(X, A) with A = W^T split along its columns.

Two ground truths are kept apart on purpose:
  * plain_*  : the unsharded definition (Y = X W^T, dX = dY W, dW = dY^T X);
  * rtp_*    : the N-step rotated computation of one worker, and ring_* the
               whole ring of N workers.
The method reaches the plain result exactly (up to the order of the sums that
cross shards), which is what the pins in tests/ check.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librtp_oracle.so")

GELU_ERF, GELU_TANH, SILU = 0, 1, 2


def _load():
    if not os.path.exists(_LIB_PATH):
        from . import build as _b
        _b.build()
    lib = ctypes.CDLL(_LIB_PATH)
    i64, dp, ci = ctypes.c_int64, ctypes.POINTER(ctypes.c_double), ctypes.c_int
    for name in ("orc_gemm_nt", "orc_gemm_nn", "orc_gemm_tn"):
        f = getattr(lib, name)
        f.argtypes = [dp, i64, dp, i64, dp, i64, i64, i64, i64, ci]
        f.restype = None
    for name in ("orc_fwd_shard", "orc_bwd_shard"):
        f = getattr(lib, name)
        f.argtypes = [ci, ci, ci]
        f.restype = ci
    lib.orc_rotations_per_pass.argtypes = [ci]
    lib.orc_rotations_per_pass.restype = ci
    lib.orc_num_threads.restype = ci
    for name in ("orc_act", "orc_act_grad"):
        f = getattr(lib, name)
        f.argtypes = [dp, dp, i64, ci]
        f.restype = None
    for name in ("orc_param_bytes", "orc_param_duplication"):
        f = getattr(lib, name)
        f.argtypes = [ci, i64, i64, i64]
        f.restype = i64
    return lib


_lib = _load()


def num_threads():
    return int(_lib.orc_num_threads())


# --------------------------------------------------------------------------
# thin wrappers: views with a last-dim stride of 1 are passed without a copy
# --------------------------------------------------------------------------

def _mat(a):
    assert a.dtype == np.float64 and a.ndim == 2 and (a.shape[1] == 1 or a.strides[1] == 8), \
        "oracle matrices are fp64, row-major, unit stride along the row"
    assert a.strides[0] % 8 == 0
    ld = a.strides[0] // 8 if a.strides[0] else max(a.shape[1], 1)
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), ld


def gemm_nt(A, B, C, accumulate=False):
    """C[m,n] (+)= sum_k A[m,k] B[n,k]."""
    M, K = A.shape
    N, K2 = B.shape
    assert K == K2 and C.shape == (M, N)
    if M == 0 or N == 0:
        return C
    (pa, lda), (pb, ldb), (pc, ldc) = _mat(A), _mat(B), _mat(C)
    _lib.orc_gemm_nt(pa, lda, pb, ldb, pc, ldc, M, N, K, int(accumulate))
    return C


def gemm_nn(A, B, C, accumulate=False):
    """C[m,n] (+)= sum_k A[m,k] B[k,n]."""
    M, K = A.shape
    K2, N = B.shape
    assert K == K2 and C.shape == (M, N)
    if M == 0 or N == 0:
        return C
    (pa, lda), (pb, ldb), (pc, ldc) = _mat(A), _mat(B), _mat(C)
    _lib.orc_gemm_nn(pa, lda, pb, ldb, pc, ldc, M, N, K, int(accumulate))
    return C


def gemm_tn(A, B, C, accumulate=False):
    """C[m,n] (+)= sum_k A[k,m] B[k,n]."""
    K, M = A.shape
    K2, N = B.shape
    assert K == K2 and C.shape == (M, N)
    if M == 0 or N == 0:
        return C
    (pa, lda), (pb, ldb), (pc, ldc) = _mat(A), _mat(B), _mat(C)
    _lib.orc_gemm_tn(pa, lda, pb, ldb, pc, ldc, M, N, K, int(accumulate))
    return C


def act(x, kind):
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    dp = ctypes.POINTER(ctypes.c_double)
    _lib.orc_act(x.ctypes.data_as(dp), y.ctypes.data_as(dp), x.size, kind)
    return y


def act_grad(x, kind):
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    dp = ctypes.POINTER(ctypes.c_double)
    _lib.orc_act_grad(x.ctypes.data_as(dp), y.ctypes.data_as(dp), x.size, kind)
    return y


# --------------------------------------------------------------------------
# schedule (Design section, workflow paragraph; Memory Arrangement paragraph)
# --------------------------------------------------------------------------

def fwd_shard(rank, step, n):
    return int(_lib.orc_fwd_shard(rank, step, n))


def bwd_shard(rank, step, n):
    return int(_lib.orc_bwd_shard(rank, step, n))


def rotations_per_pass(n):
    return int(_lib.orc_rotations_per_pass(n))


def shard_rows(k, O, n):
    """Half-open range of the output features that make up shard k."""
    assert O % n == 0, "the partition factor must divide the partitioned dimension"
    o = O // n
    return k * o, (k + 1) * o


# --------------------------------------------------------------------------
# plain (unsharded) definitions
# --------------------------------------------------------------------------

def plain_linear_fwd(X, W, b=None):
    """Y = X W^T (+ b on every row)."""
    T, _ = X.shape
    O, _ = W.shape
    Y = gemm_nt(X, W, np.empty((T, O)))
    if b is not None:
        for t in range(T):
            Y[t, :] += b
    return Y


def plain_linear_bwd(X, W, dY):
    """Returns (dX, dW) = (dY W, dY^T X)."""
    T, I = X.shape
    O, _ = W.shape
    dX = gemm_nn(dY, W, np.empty((T, I)))
    dW = gemm_tn(dY, X, np.empty((O, I)))
    return dX, dW


def plain_bias_grad(dY):
    """db[j] = sum over tokens of dY[t, j]."""
    T, O = dY.shape
    db = np.zeros(O)
    for t in range(T):
        db += dY[t, :]
    return db


def plain_mlp(X, W1, W2, dY, kind=GELU_ERF, b1=None, b2=None):
    """MLP block: a GEMM, the nonlinearity, a second GEMM (RTP Transformers
    section, linear-block item), each with an optional bias.  Returns a dict
    of every tensor."""
    Z = plain_linear_fwd(X, W1, b1)
    H = act(Z, kind)
    Y = plain_linear_fwd(H, W2, b2)
    dH, dW2 = plain_linear_bwd(H, W2, dY)
    dZ = dH * act_grad(Z, kind)
    dX, dW1 = plain_linear_bwd(X, W1, dZ)
    return dict(Z=Z, H=H, Y=Y, dH=dH, dZ=dZ, dX=dX, dW1=dW1, dW2=dW2, db1=plain_bias_grad(dZ), db2=plain_bias_grad(dY))


def plain_swiglu(X, Wg, Wu, Wd, dY, bg=None, bu=None, bd=None):
    """Gated MLP: H = silu(X Wg^T + bg) * (X Wu^T + bu), Y = H Wd^T + bd, and its gradients (biases optional)."""
    A = plain_linear_fwd(X, Wg, bg)
    B = plain_linear_fwd(X, Wu, bu)
    sA = act(A, SILU)
    H = sA * B
    Y = plain_linear_fwd(H, Wd, bd)
    dH, dWd = plain_linear_bwd(H, Wd, dY)
    dA = dH * B * act_grad(A, SILU)
    dB = dH * sA
    dXa, dWg = plain_linear_bwd(X, Wg, dA)
    dXb, dWu = plain_linear_bwd(X, Wu, dB)
    return dict(A=A, B=B, H=H, Y=Y, dH=dH, dA=dA, dB=dB, dX=dXa + dXb, dWg=dWg, dWu=dWu, dWd=dWd,
                dbg=plain_bias_grad(dA), dbu=plain_bias_grad(dB), dbd=plain_bias_grad(dY))


# --------------------------------------------------------------------------
# one worker's rotated pass
# --------------------------------------------------------------------------

class _Ring:
    """The shard store one worker sees: `home[k]` stands for the memory of
    the other workers, `resident` is the shard being computed on and
    `staging` is the communication buffer of the out-of-place variant
    (Rotating Communication Primitive section).  Every move is a copy."""

    def __init__(self, w_shards, g_shards, rank):
        self.n = len(w_shards)
        self.rank = rank
        self.home_w = [w.copy() for w in w_shards]
        self.home_g = [g.copy() for g in g_shards]
        self.res_id = rank
        self.res_w = self.home_w[rank].copy()
        self.res_g = self.home_g[rank].copy()
        self.stage_w = np.full_like(self.res_w, np.nan)
        self.stage_g = np.full_like(self.res_g, np.nan)
        self.sent, self.received = [], []

    def begin_backward(self):
        """Gradient shards come into being where the weights ended the
        forward pass: the worker now holds the gradient shard that belongs to
        the weight shard it holds."""
        np.copyto(self.res_g, self.home_g[self.res_id])

    def rotate(self, incoming, with_grad):
        """Pass the resident shard on and take shard `incoming` in."""
        k = self.res_id
        # receive into the staging buffer ...
        np.copyto(self.stage_w, self.home_w[incoming])
        if with_grad:
            np.copyto(self.stage_g, self.home_g[incoming])
        # ... send the held shard to its next holder ...
        np.copyto(self.home_w[k], self.res_w)
        if with_grad:
            np.copyto(self.home_g[k], self.res_g)
        self.sent.append(k)
        self.received.append(incoming)
        # ... and swap the roles of the two buffers.
        self.res_w, self.stage_w = self.stage_w, self.res_w
        if with_grad:
            self.res_g, self.stage_g = self.stage_g, self.res_g
        self.res_id = incoming


def _split_rows(W, n):
    O = W.shape[0]
    return [W[slice(*shard_rows(k, O, n))] for k in range(n)]


def _split_cols(W, n):
    C = W.shape[1]
    return [np.ascontiguousarray(W[:, slice(*shard_rows(k, C, n))]) for k in range(n)]


def rtp_linear_out(X, W, dY, n, rank, G0=None):
    """Output-partitioned linear, one worker, forward then backward.

    Shard k is rows [k o, (k+1) o) of W.  Forward step t computes on shard
    (rank - t) mod n and writes the matching column slice of Y (the concat of
    the paper folded into the store); backward step s computes on shard
    (rank + 1 + s) mod n, adds dY_k^T X onto the gradient shard that travels
    with that weight and adds dY_k W_k onto dX.  G0 is what the gradient
    shards hold when they arrive (zeros if omitted).
    """
    T, I = X.shape
    O = W.shape[0]
    if G0 is None:
        G0 = np.zeros((O, I))
    ring = _Ring(_split_rows(W, n), _split_rows(G0, n), rank)
    Y = np.full((T, O), np.nan)
    fwd_log, bwd_log = [], []
    for t in range(n):
        k = ring.res_id
        assert k == fwd_shard(rank, t, n)
        lo, hi = shard_rows(k, O, n)
        gemm_nt(X, ring.res_w, Y[:, lo:hi])
        fwd_log.append((t, k))
        if t < n - 1:
            ring.rotate((k - 1) % n, with_grad=False)
    res_after_fwd = ring.res_id
    n_fwd_rot = len(ring.sent)

    dX = np.zeros((T, I))
    ring.begin_backward()
    for s in range(n):
        k = ring.res_id
        assert k == bwd_shard(rank, s, n)
        lo, hi = shard_rows(k, O, n)
        gemm_tn(dY[:, lo:hi], X, ring.res_g, accumulate=True)
        gemm_nn(dY[:, lo:hi], ring.res_w, dX, accumulate=True)
        bwd_log.append((s, k))
        if s < n - 1:
            ring.rotate((k + 1) % n, with_grad=True)
    # leave the worker's own shard where a reader of the store expects it
    G = [g.copy() for g in ring.home_g]
    G[ring.res_id] = ring.res_g.copy()
    Wback = [w.copy() for w in ring.home_w]
    Wback[ring.res_id] = ring.res_w.copy()
    return dict(Y=Y, dX=dX, G=np.concatenate(G, axis=0), W_after=np.concatenate(Wback, axis=0),
                fwd_log=fwd_log, bwd_log=bwd_log, resident_after_fwd=res_after_fwd,
                resident_after_bwd=ring.res_id, fwd_rotations=n_fwd_rot,
                bwd_rotations=len(ring.sent) - n_fwd_rot, sent=ring.sent, received=ring.received)


def rtp_linear_out_bias(X, W, b, dY, n, rank, G0=None, gb0=None):
    """Output-partitioned linear with a bias that rides in the same shard as its rows of W (the flat
    parameter of the FlatParameter section holds every parameter of the unit).  Row j of the shard is
    (W[j, :], b[j]); the step's product with (X, 1) gives X W_k^T + b_k, and the travelling gradient
    shard collects (dY_k^T X, dY_k^T 1) in the same layout.  Returns the dict of rtp_linear_out with
    G split into G (matrix part) and gb (bias part)."""
    T, I = X.shape
    O = W.shape[0]
    Wa = np.concatenate((W, np.asarray(b, dtype=np.float64).reshape(O, 1)), axis=1)
    Xa = np.concatenate((X, np.ones((T, 1))), axis=1)
    Ga = np.concatenate((np.zeros((O, I)) if G0 is None else G0,
                         (np.zeros(O) if gb0 is None else np.asarray(gb0, dtype=np.float64)).reshape(O, 1)), axis=1)
    out = rtp_linear_out(np.ascontiguousarray(Xa), np.ascontiguousarray(Wa), dY, n, rank, np.ascontiguousarray(Ga))
    out["dX"] = np.ascontiguousarray(out["dX"][:, :I])      # the constant 1 has no gradient
    out["gb"] = np.ascontiguousarray(out["G"][:, I])
    out["G"] = np.ascontiguousarray(out["G"][:, :I])
    out["b_after"] = np.ascontiguousarray(out["W_after"][:, I])
    out["W_after"] = np.ascontiguousarray(out["W_after"][:, :I])
    return out


def bias_pieces(O, n):
    """The bias of an input-partitioned layer is not partitioned by the layer's
    own split; the flat parameter spreads it evenly over the N shards
    (FlatParameter paragraph): piece k = entries [k p, (k+1) p) of b with
    p = ceil(O / N), the last pieces short or empty."""
    p = -(-O // n)
    return [(min(k * p, O), min((k + 1) * p, O)) for k in range(n)]


def _padded_pieces(v, pieces):
    """The pieces of a vector as equal-sized arrays, the short ones padded with zeros (the flat
    parameter's padding): every shard of the ring has the same size."""
    p = max(hi - lo for lo, hi in pieces)
    out = []
    for lo, hi in pieces:
        a = np.zeros(p)
        a[:hi - lo] = v[lo:hi]
        out.append(a)
    return out


def _unpad_pieces(arrs, pieces):
    return np.concatenate([a[:hi - lo] for a, (lo, hi) in zip(arrs, pieces)])


def rtp_linear_in(Xin, W, dY, n, rank, G0=None, b=None, gb0=None):
    """Input-partitioned linear (the layer that follows a column-partitioned
    one: Partition Strategies section, second item).  Shard k is columns
    [k o, (k+1) o) of W[O, I]; forward sums the N partial products into Y,
    backward writes the matching column slice of dXin and adds dY^T Xin_k
    onto the travelling gradient shard.  With a bias, shard k also carries
    piece k of b (bias_pieces): its step adds the piece to its entries of every
    output row, and in the backward pass the piece's gradient (column sums of
    dY) is added onto the piece of the travelling gradient shard."""
    T, I = Xin.shape
    O = W.shape[0]
    if G0 is None:
        G0 = np.zeros((O, I))
    ring = _Ring(_split_cols(W, n), _split_cols(G0, n), rank)
    pieces = bias_pieces(O, n)
    if b is not None:
        b = np.asarray(b, dtype=np.float64)
        gb0 = np.zeros(O) if gb0 is None else np.asarray(gb0, dtype=np.float64)
        bring = _Ring(_padded_pieces(b, pieces), _padded_pieces(gb0, pieces), rank)
    Y = np.zeros((T, O))
    fwd_log, bwd_log = [], []
    for t in range(n):
        k = ring.res_id
        assert k == fwd_shard(rank, t, n)
        lo, hi = shard_rows(k, I, n)
        gemm_nt(Xin[:, lo:hi], ring.res_w, Y, accumulate=True)
        if b is not None:
            assert bring.res_id == k
            plo, phi = pieces[k]
            for row in range(T):
                Y[row, plo:phi] += bring.res_w[:phi - plo]
        fwd_log.append((t, k))
        if t < n - 1:
            ring.rotate((k - 1) % n, with_grad=False)
            if b is not None:
                bring.rotate((k - 1) % n, with_grad=False)
    res_after_fwd = ring.res_id
    dXin = np.full((T, I), np.nan)
    ring.begin_backward()
    if b is not None:
        bring.begin_backward()
    for s in range(n):
        k = ring.res_id
        assert k == bwd_shard(rank, s, n)
        lo, hi = shard_rows(k, I, n)
        gemm_tn(dY, Xin[:, lo:hi], ring.res_g, accumulate=True)
        gemm_nn(dY, ring.res_w, dXin[:, lo:hi])
        if b is not None:
            assert bring.res_id == k
            plo, phi = pieces[k]
            bring.res_g[:phi - plo] += plain_bias_grad(np.ascontiguousarray(dY[:, plo:phi]))
        bwd_log.append((s, k))
        if s < n - 1:
            ring.rotate((k + 1) % n, with_grad=True)
            if b is not None:
                bring.rotate((k + 1) % n, with_grad=True)
    G = [g.copy() for g in ring.home_g]
    G[ring.res_id] = ring.res_g.copy()
    Wback = [w.copy() for w in ring.home_w]
    Wback[ring.res_id] = ring.res_w.copy()
    out = dict(Y=Y, dX=dXin, G=np.concatenate(G, axis=1), W_after=np.concatenate(Wback, axis=1),
               fwd_log=fwd_log, bwd_log=bwd_log, resident_after_fwd=res_after_fwd,
               resident_after_bwd=ring.res_id)
    if b is not None:
        gb = [g.copy() for g in bring.home_g]
        gb[bring.res_id] = bring.res_g.copy()
        bb = [w.copy() for w in bring.home_w]
        bb[bring.res_id] = bring.res_w.copy()
        out["gb"] = _unpad_pieces(gb, pieces)
        out["b_after"] = _unpad_pieces(bb, pieces)
    return out


def rtp_mlp(X, W1, W2, dY, n, rank, kind=GELU_ERF, G1_0=None, G2_0=None, b1=None, b2=None, gb1_0=None, gb2_0=None):
    """MLP block with W1 output-partitioned and W2 input-partitioned, so that
    unit k = (rows k of W1, columns k of W2) is self-contained and the two
    shards rotate as one message (the FlatParameter idea).  Step order is the
    rotation schedule; inside a step the order is the chain rule's.  Optional
    biases (both or none): b1's entries ride with their rows of W1, b2 is
    spread over the shards in pieces (bias_pieces)."""
    T, I = X.shape
    O1 = W1.shape[0]
    O2 = W2.shape[0]
    G1_0 = np.zeros_like(W1) if G1_0 is None else G1_0
    G2_0 = np.zeros_like(W2) if G2_0 is None else G2_0
    r1 = _Ring(_split_rows(W1, n), _split_rows(G1_0, n), rank)
    r2 = _Ring(_split_cols(W2, n), _split_cols(G2_0, n), rank)
    rings = [r1, r2]
    biased = b1 is not None
    assert biased == (b2 is not None)
    if biased:
        b1, b2 = np.asarray(b1, dtype=np.float64), np.asarray(b2, dtype=np.float64)
        gb1_0 = np.zeros(O1) if gb1_0 is None else np.asarray(gb1_0, dtype=np.float64)
        gb2_0 = np.zeros(O2) if gb2_0 is None else np.asarray(gb2_0, dtype=np.float64)
        rows = [shard_rows(k, O1, n) for k in range(n)]
        pieces = bias_pieces(O2, n)
        rb1 = _Ring([b1[lo:hi].copy() for lo, hi in rows], [gb1_0[lo:hi].copy() for lo, hi in rows], rank)
        rb2 = _Ring(_padded_pieces(b2, pieces), _padded_pieces(gb2_0, pieces), rank)
        rings += [rb1, rb2]
    Z = np.full((T, O1), np.nan)
    H = np.full((T, O1), np.nan)
    Y = np.zeros((T, O2))
    for t in range(n):
        k = r1.res_id
        assert all(r_.res_id == k for r_ in rings) and k == fwd_shard(rank, t, n)
        lo, hi = shard_rows(k, O1, n)
        gemm_nt(X, r1.res_w, Z[:, lo:hi])
        if biased:
            for row in range(T):
                Z[row, lo:hi] += rb1.res_w
        H[:, lo:hi] = act(Z[:, lo:hi], kind)
        gemm_nt(np.ascontiguousarray(H[:, lo:hi]), r2.res_w, Y, accumulate=True)
        if biased:
            plo, phi = pieces[k]
            for row in range(T):
                Y[row, plo:phi] += rb2.res_w[:phi - plo]
        if t < n - 1:
            for r_ in rings:
                r_.rotate((k - 1) % n, with_grad=False)
    dX = np.zeros((T, I))
    for r_ in rings:
        r_.begin_backward()
    for s in range(n):
        k = r1.res_id
        assert all(r_.res_id == k for r_ in rings) and k == bwd_shard(rank, s, n)
        lo, hi = shard_rows(k, O1, n)
        Hk = np.ascontiguousarray(H[:, lo:hi])
        gemm_tn(dY, Hk, r2.res_g, accumulate=True)
        if biased:
            plo, phi = pieces[k]
            rb2.res_g[:phi - plo] += plain_bias_grad(np.ascontiguousarray(dY[:, plo:phi]))
        dHk = gemm_nn(dY, r2.res_w, np.empty((T, hi - lo)))
        dZk = dHk * act_grad(Z[:, lo:hi], kind)
        gemm_tn(dZk, X, r1.res_g, accumulate=True)
        if biased:
            rb1.res_g += plain_bias_grad(dZk)
        gemm_nn(dZk, r1.res_w, dX, accumulate=True)
        if s < n - 1:
            for r_ in rings:
                r_.rotate((k + 1) % n, with_grad=True)

    def gather(ring, axis):
        g = [x.copy() for x in ring.home_g]
        g[ring.res_id] = ring.res_g.copy()
        return np.concatenate(g, axis=axis)

    out = dict(Z=Z, H=H, Y=Y, dX=dX, dW1=gather(r1, 0), dW2=gather(r2, 1), resident_after_bwd=r1.res_id)
    if biased:
        g2 = [x.copy() for x in rb2.home_g]
        g2[rb2.res_id] = rb2.res_g.copy()
        out["db1"], out["db2"] = gather(rb1, 0), _unpad_pieces(g2, pieces)
    return out


def rtp_swiglu(X, Wg, Wu, Wd, dY, n, rank, Gg0=None, Gu0=None, Gd0=None, bg=None, bu=None, bd=None,
               gbg0=None, gbu0=None, gbd0=None):
    """Gated MLP with gate and up output-partitioned and down
    input-partitioned; unit k = (gate_k, up_k, down_k).  Optional biases (all
    three or none), carried as in rtp_mlp: the gate's and the up matrix's
    entries ride with their rows, the down matrix's is spread in pieces."""
    T, I = X.shape
    O1 = Wg.shape[0]
    O2 = Wd.shape[0]
    Gg0 = np.zeros_like(Wg) if Gg0 is None else Gg0
    Gu0 = np.zeros_like(Wu) if Gu0 is None else Gu0
    Gd0 = np.zeros_like(Wd) if Gd0 is None else Gd0
    rg = _Ring(_split_rows(Wg, n), _split_rows(Gg0, n), rank)
    ru = _Ring(_split_rows(Wu, n), _split_rows(Gu0, n), rank)
    rd = _Ring(_split_cols(Wd, n), _split_cols(Gd0, n), rank)
    rings = [rg, ru, rd]
    biased = bg is not None
    assert biased == (bu is not None) == (bd is not None)
    if biased:
        vec = lambda v, size: np.zeros(size) if v is None else np.asarray(v, dtype=np.float64)
        bg, bu, bd = vec(bg, O1), vec(bu, O1), vec(bd, O2)
        gbg0, gbu0, gbd0 = vec(gbg0, O1), vec(gbu0, O1), vec(gbd0, O2)
        rows = [shard_rows(k, O1, n) for k in range(n)]
        pieces = bias_pieces(O2, n)
        rbg = _Ring([bg[lo:hi].copy() for lo, hi in rows], [gbg0[lo:hi].copy() for lo, hi in rows], rank)
        rbu = _Ring([bu[lo:hi].copy() for lo, hi in rows], [gbu0[lo:hi].copy() for lo, hi in rows], rank)
        rbd = _Ring(_padded_pieces(bd, pieces), _padded_pieces(gbd0, pieces), rank)
        rings += [rbg, rbu, rbd]
    A = np.full((T, O1), np.nan)
    B = np.full((T, O1), np.nan)
    H = np.full((T, O1), np.nan)
    Y = np.zeros((T, O2))
    for t in range(n):
        k = rg.res_id
        assert all(r_.res_id == k for r_ in rings) and k == fwd_shard(rank, t, n)
        lo, hi = shard_rows(k, O1, n)
        gemm_nt(X, rg.res_w, A[:, lo:hi])
        gemm_nt(X, ru.res_w, B[:, lo:hi])
        if biased:
            for row in range(T):
                A[row, lo:hi] += rbg.res_w
                B[row, lo:hi] += rbu.res_w
        H[:, lo:hi] = act(A[:, lo:hi], SILU) * B[:, lo:hi]
        gemm_nt(np.ascontiguousarray(H[:, lo:hi]), rd.res_w, Y, accumulate=True)
        if biased:
            plo, phi = pieces[k]
            for row in range(T):
                Y[row, plo:phi] += rbd.res_w[:phi - plo]
        if t < n - 1:
            for r_ in rings:
                r_.rotate((k - 1) % n, with_grad=False)
    dX = np.zeros((T, I))
    for r_ in rings:
        r_.begin_backward()
    for s in range(n):
        k = rg.res_id
        assert all(r_.res_id == k for r_ in rings) and k == bwd_shard(rank, s, n)
        lo, hi = shard_rows(k, O1, n)
        Hk = np.ascontiguousarray(H[:, lo:hi])
        gemm_tn(dY, Hk, rd.res_g, accumulate=True)
        if biased:
            plo, phi = pieces[k]
            rbd.res_g[:phi - plo] += plain_bias_grad(np.ascontiguousarray(dY[:, plo:phi]))
        dHk = gemm_nn(dY, rd.res_w, np.empty((T, hi - lo)))
        dAk = dHk * B[:, lo:hi] * act_grad(A[:, lo:hi], SILU)
        dBk = dHk * act(A[:, lo:hi], SILU)
        gemm_tn(dAk, X, rg.res_g, accumulate=True)
        gemm_tn(dBk, X, ru.res_g, accumulate=True)
        if biased:
            rbg.res_g += plain_bias_grad(dAk)
            rbu.res_g += plain_bias_grad(dBk)
        gemm_nn(dAk, rg.res_w, dX, accumulate=True)
        gemm_nn(dBk, ru.res_w, dX, accumulate=True)
        if s < n - 1:
            for r_ in rings:
                r_.rotate((k + 1) % n, with_grad=True)

    def gather(ring, axis):
        g = [x.copy() for x in ring.home_g]
        g[ring.res_id] = ring.res_g.copy()
        return np.concatenate(g, axis=axis)

    out = dict(A=A, B=B, H=H, Y=Y, dX=dX, dWg=gather(rg, 0), dWu=gather(ru, 0), dWd=gather(rd, 1),
               resident_after_bwd=rg.res_id)
    if biased:
        gd = [x.copy() for x in rbd.home_g]
        gd[rbd.res_id] = rbd.res_g.copy()
        out["dbg"], out["dbu"], out["dbd"] = gather(rbg, 0), gather(rbu, 0), _unpad_pieces(gd, pieces)
    return out


# --------------------------------------------------------------------------
# expert partition (Partition Strategies section, last item; RTP Transformers
# section, MoE block item)
# --------------------------------------------------------------------------
# Worker r starts with expert r; the experts rotate like any other shard, and
# at each step the worker runs the expert it holds on those of its own tokens
# that are routed to it; the outputs of the N steps, put back in token order
# ("concatenation"), are the layer's output.  No token leaves the worker.
# The paper defines no router: the routing (one expert per token) is an input.

def moe_dispatch(route, n, align=1):
    """Groups token indices by expert, token order kept inside a group
    (a stable grouping), each group starting at a multiple of `align` rows.
    Returns (counts[n], begin[n+1], perm) with perm[p] = the token held by
    grouped row p, or -1 for a padding row; begin[n] = len(perm)."""
    route = [int(e) for e in route]
    counts = [0] * n
    for e in route:
        assert 0 <= e < n, "route holds expert ids"
        counts[e] += 1
    begin = [0]
    for e in range(n):
        begin.append(begin[-1] + (counts[e] + align - 1) // align * align)
    perm = [-1] * begin[n]
    fill = list(begin[:n])
    for t, e in enumerate(route):
        perm[fill[e]] = t
        fill[e] += 1
    return counts, begin, perm


def _expert_fwd(X, W, kind, gated):
    """One expert on the rows of X: returns (pre-activations, hidden, output)."""
    if gated:
        Wg, Wu, Wd = W
        A, Bm = plain_linear_fwd(X, Wg), plain_linear_fwd(X, Wu)
        H = act(A, SILU) * Bm
        return (A, Bm), H, plain_linear_fwd(H, Wd)
    W1, W2 = W
    Z = plain_linear_fwd(X, W1)
    H = act(Z, kind)
    return (Z,), H, plain_linear_fwd(H, W2)


def _expert_bwd(X, W, pre, H, dY, G, kind, gated):
    """Chain rule through one expert: adds the weight gradients onto the
    arrays of G and returns the gradient of the expert's input rows."""
    Tm, I = X.shape
    if gated:
        Wg, Wu, Wd = W
        A, Bm = pre
        gemm_tn(dY, H, G[2], accumulate=True)
        dH = gemm_nn(dY, Wd, np.empty_like(H))
        dA = dH * Bm * act_grad(A, SILU)
        dB = dH * act(A, SILU)
        gemm_tn(dA, X, G[0], accumulate=True)
        gemm_tn(dB, X, G[1], accumulate=True)
        dX = gemm_nn(dA, Wg, np.empty((Tm, I)))
        return gemm_nn(dB, Wu, dX, accumulate=True)
    W1, W2 = W
    (Z,) = pre
    gemm_tn(dY, H, G[1], accumulate=True)
    dH = gemm_nn(dY, W2, np.empty_like(H))
    dZ = dH * act_grad(Z, kind)
    gemm_tn(dZ, X, G[0], accumulate=True)
    return gemm_nn(dZ, W1, np.empty((Tm, I)))


def plain_moe(X, route, experts, dY, kind=GELU_ERF, G0=None):
    """The definition, token by token: token t goes through expert route[t]
    and nothing else.  `experts[e]` is (W1, W2) or (Wg, Wu, Wd); G0 the
    gradients to accumulate onto (same structure).  Returns Y, dX and the
    per-expert weight gradients."""
    T, I = X.shape
    gated = len(experts[0]) == 3
    O2 = experts[0][-1].shape[0]
    G = [[np.zeros_like(w) for w in ex] for ex in experts] if G0 is None else [[g.copy() for g in ex] for ex in G0]
    Y = np.full((T, O2), np.nan)
    dX = np.full((T, I), np.nan)
    for t in range(T):
        e = int(route[t])
        x = np.ascontiguousarray(X[t:t + 1])
        pre, H, y = _expert_fwd(x, experts[e], kind, gated)
        Y[t] = y[0]
        dX[t] = _expert_bwd(x, experts[e], pre, H, np.ascontiguousarray(dY[t:t + 1]), G[e], kind, gated)[0]
    return dict(Y=Y, dX=dX, G=G)


def rtp_moe(X, route, experts, dY, n, rank, kind=GELU_ERF, G0=None):
    """Expert rotation on one worker: N steps forward (clockwise), N steps
    backward (counter-clockwise, each expert's gradients travelling with it).
    The shard of the ring is one whole expert."""
    T, I = X.shape
    assert len(experts) == n
    gated = len(experts[0]) == 3
    O2 = experts[0][-1].shape[0]
    G0 = [[np.zeros_like(w) for w in ex] for ex in experts] if G0 is None else G0
    nm = len(experts[0])
    rings = [_Ring([experts[e][j] for e in range(n)], [G0[e][j] for e in range(n)], rank) for j in range(nm)]
    counts, begin, perm = moe_dispatch(route, n)
    Y = np.full((T, O2), np.nan)
    saved = {}
    fwd_log, bwd_log = [], []
    for t in range(n):
        e = rings[0].res_id
        assert e == fwd_shard(rank, t, n)
        rows = perm[begin[e]:begin[e + 1]]
        fwd_log.append((t, e, len(rows)))
        if rows:                                   # an expert without tokens only passes through
            Xe = np.ascontiguousarray(X[rows]).reshape(len(rows), I)
            pre, H, Ye = _expert_fwd(Xe, [r_.res_w for r_ in rings], kind, gated)
            Y[rows] = Ye
            saved[e] = (Xe, pre, H)
        if t < n - 1:
            for r_ in rings:
                r_.rotate((e - 1) % n, with_grad=False)
    dX = np.full((T, I), np.nan)
    for r_ in rings:
        r_.begin_backward()
    for s in range(n):
        e = rings[0].res_id
        assert e == bwd_shard(rank, s, n)
        rows = perm[begin[e]:begin[e + 1]]
        bwd_log.append((s, e, len(rows)))
        if rows:
            Xe, pre, H = saved[e]
            dYe = np.ascontiguousarray(dY[rows]).reshape(len(rows), O2)
            dX[rows] = _expert_bwd(Xe, [r_.res_w for r_ in rings], pre, H, dYe, [r_.res_g for r_ in rings], kind,
                                   gated)
        if s < n - 1:
            for r_ in rings:
                r_.rotate((e + 1) % n, with_grad=True)
    G = []
    for e in range(n):
        G.append([(r_.res_g if r_.res_id == e else r_.home_g[e]).copy() for r_ in rings])
    return dict(Y=Y, dX=dX, G=G, counts=counts, begin=begin, perm=perm, fwd_log=fwd_log, bwd_log=bwd_log,
                resident_after_bwd=rings[0].res_id)


# --------------------------------------------------------------------------
# the whole ring of N workers (tiny shapes only)
# --------------------------------------------------------------------------

def ring_linear_out(X, W, dY, n):
    """All N workers of an output-partitioned linear.  X and dY are the
    global batch; worker r owns rows [r T/n, (r+1) T/n).  At every step the
    map worker -> held shard must be a bijection, every send must be matched
    by the neighbour's receive, and at the end each gradient shard, back at
    its owner, must hold the sum over all workers (the travelling gradient is
    the reduction).  Returns the assembled Y, dX, dW and the traffic log."""
    Tg, I = X.shape
    O = W.shape[0]
    assert Tg % n == 0
    Tl = Tg // n
    o = O // n
    Xr = [X[r * Tl:(r + 1) * Tl] for r in range(n)]
    dYr = [dY[r * Tl:(r + 1) * Tl] for r in range(n)]
    held_w = [W[r * o:(r + 1) * o].copy() for r in range(n)]   # worker r starts with shard r
    held_g = [np.zeros((o, I)) for _ in range(n)]
    held_id = list(range(n))
    Y = [np.full((Tl, O), np.nan) for _ in range(n)]
    dX = [np.zeros((Tl, I)) for _ in range(n)]
    sends = [[] for _ in range(n)]
    recvs = [[] for _ in range(n)]
    history = []

    def rotate(direction, with_grad):
        # direction +1: worker r sends to r+1 and receives from r-1 (forward);
        # direction -1: the mirror image (backward).
        nonlocal held_w, held_g, held_id
        new_w, new_g, new_id = [None] * n, [None] * n, [None] * n
        for r in range(n):
            dst = (r + direction) % n
            new_w[dst] = held_w[r]
            new_g[dst] = held_g[r] if with_grad else None
            new_id[dst] = held_id[r]
            sends[r].append(held_id[r])
            recvs[dst].append(held_id[r])
        if not with_grad:
            new_g = held_g  # gradient shards do not exist yet in the forward pass
        held_w, held_g, held_id = new_w, new_g, new_id

    for t in range(n):
        assert sorted(held_id) == list(range(n)), "held shards must be a bijection"
        history.append(("fwd", t, tuple(held_id)))
        for r in range(n):
            k = held_id[r]
            assert k == fwd_shard(r, t, n)
            gemm_nt(Xr[r], held_w[r], Y[r][:, k * o:(k + 1) * o])
        if t < n - 1:
            rotate(+1, with_grad=False)
    # gradient shards are created where the weights ended the forward pass
    held_g = [np.zeros((o, I)) for _ in range(n)]
    for s in range(n):
        assert sorted(held_id) == list(range(n))
        history.append(("bwd", s, tuple(held_id)))
        for r in range(n):
            k = held_id[r]
            assert k == bwd_shard(r, s, n)
            gemm_tn(dYr[r][:, k * o:(k + 1) * o], Xr[r], held_g[r], accumulate=True)
            gemm_nn(dYr[r][:, k * o:(k + 1) * o], held_w[r], dX[r], accumulate=True)
        if s < n - 1:
            rotate(-1, with_grad=True)
    assert held_id == list(range(n)), "every shard must be back with its owner"
    return dict(Y=np.concatenate(Y, axis=0), dX=np.concatenate(dX, axis=0),
                dW=np.concatenate(held_g, axis=0), W_after=np.concatenate(held_w, axis=0),
                sends=sends, recvs=recvs, history=history)


# --------------------------------------------------------------------------
# parameter memory (Table 1)
# --------------------------------------------------------------------------

TECHNIQUES = dict(none=0, tensor_parallel=1, data_parallel=2, pipeline_parallel=3, fsdp=4,
                  rtp=5, rtp_inplace=6)


def param_bytes(technique, W, G, n):
    """System-wide parameter memory of Table 1 for W weight bytes and G
    gradient bytes."""
    return int(_lib.orc_param_bytes(TECHNIQUES[technique], W, G, n))


def param_duplication(technique, W, G, n):
    return int(_lib.orc_param_duplication(TECHNIQUES[technique], W, G, n))


def worker_param_bytes(technique, W, G, n):
    """One worker's even share of the system-wide figure."""
    total = param_bytes(technique, W, G, n)
    assert total % n == 0
    return total // n
