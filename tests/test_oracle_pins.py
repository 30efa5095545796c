"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix, never against itself.  CPU only."""
import os

import numpy as np
import pytest

import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng_mats(seed, T, I, O):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((T, I)), rng.standard_normal((O, I)), rng.standard_normal((T, O))


# ---------------------------------------------------------------- schedule --

@pytest.mark.parametrize("n", list(range(1, 65)))
def test_schedule_invariants_exhaustive(n):
    """Workflow paragraph of the Design section: N computes and N-1 rotations
    per pass; forward ends on the next worker's shard, backward ends on the
    worker's own; every shard is visited exactly once per pass."""
    assert orc.rotations_per_pass(n) == n - 1
    for r in range(n):
        f = [orc.fwd_shard(r, t, n) for t in range(n)]
        b = [orc.bwd_shard(r, s, n) for s in range(n)]
        assert f[0] == r
        assert sorted(f) == list(range(n)) and sorted(b) == list(range(n))
        assert f[-1] == (r + 1) % n if n > 1 else f[-1] == r
        assert b[0] == f[-1], "backward starts on the shard forward ended on"
        assert b[-1] == r, "the worker recovers its own shard"
        for t in range(1, n):
            assert f[t] == (f[t - 1] - 1) % n      # receives from the previous worker
            assert b[t] == (b[t - 1] + 1) % n      # mirror image
    # at every step the map worker -> shard is a bijection (each worker sends one, receives one)
    for t in range(n):
        assert sorted(orc.fwd_shard(r, t, n) for r in range(n)) == list(range(n))
        assert sorted(orc.bwd_shard(r, t, n) for r in range(n)) == list(range(n))
    # what r holds at step t+1 is what r-1 held at step t (send to next, receive from previous)
    for r in range(n):
        for t in range(n - 1):
            assert orc.fwd_shard(r, t + 1, n) == orc.fwd_shard((r - 1) % n, t, n)
            assert orc.bwd_shard(r, t + 1, n) == orc.bwd_shard((r + 1) % n, t, n)


def test_two_worker_example_from_the_paper():
    """Two workers, as in the paper's overview figure text: worker 1 computes
    on its own shard, then on worker 2's... in our 0-based ranks the forward
    of worker 0 sees shards 0 then 1, and ends holding the subsequent worker's
    shard."""
    assert [orc.fwd_shard(0, t, 2) for t in range(2)] == [0, 1]
    assert [orc.fwd_shard(1, t, 2) for t in range(2)] == [1, 0]
    assert [orc.bwd_shard(0, s, 2) for s in range(2)] == [1, 0]


def test_block_identity_fixture():
    """The printed 2-worker block equation: block (i, j) of Y is GEMM(X_i, A_j)."""
    rows = []
    with open(os.path.join(GOLDEN, "two_worker_block_identity.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            lhs, rhs = line.split("->")
            rows.append(tuple(int(v) - 1 for v in lhs.split() + rhs.split()))
    X, W, dY = rng_mats(3, 6, 5, 8)
    res = orc.ring_linear_out(X, W, dY, 2)
    Tl, o = 3, 4
    for (i, j, xi, aj) in rows:
        want = X[xi * Tl:(xi + 1) * Tl] @ W[aj * o:(aj + 1) * o].T
        np.testing.assert_allclose(res["Y"][i * Tl:(i + 1) * Tl, j * o:(j + 1) * o], want, rtol=0, atol=1e-13)


# ------------------------------------------------------------ contractions --

def brute(X, W, dY):
    """Independent statement: different loop nest, extended precision."""
    T, I = X.shape
    O = W.shape[0]
    ld = np.longdouble
    Y = np.zeros((T, O), dtype=ld)
    dX = np.zeros((T, I), dtype=ld)
    dW = np.zeros((O, I), dtype=ld)
    for i in range(I):
        for j in range(O):
            for t in range(T):
                Y[t, j] += ld(X[t, i]) * ld(W[j, i])
                dX[t, i] += ld(dY[t, j]) * ld(W[j, i])
                dW[j, i] += ld(dY[t, j]) * ld(X[t, i])
    return Y.astype(np.float64), dX.astype(np.float64), dW.astype(np.float64)


@pytest.mark.parametrize("T,I,O", [(1, 1, 1), (2, 3, 4), (5, 7, 12), (3, 2, 6), (4, 5, 1)])
def test_plain_vs_brute_force(T, I, O):
    X, W, dY = rng_mats(T * 100 + I * 10 + O, T, I, O)
    Yb, dXb, dWb = brute(X, W, dY)
    np.testing.assert_allclose(orc.plain_linear_fwd(X, W), Yb, rtol=0, atol=1e-13)
    dX, dW = orc.plain_linear_bwd(X, W, dY)
    np.testing.assert_allclose(dX, dXb, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dW, dWb, rtol=0, atol=1e-13)


@pytest.mark.parametrize("T,I,O", [(17, 33, 40), (64, 256, 512), (130, 70, 96)])
def test_plain_vs_library_matmul(T, I, O):
    """Special case that reduces to a library routine: numpy's fp64 matmul."""
    X, W, dY = rng_mats(7, T, I, O)
    np.testing.assert_allclose(orc.plain_linear_fwd(X, W), X @ W.T, rtol=0, atol=1e-11)
    dX, dW = orc.plain_linear_bwd(X, W, dY)
    np.testing.assert_allclose(dX, dY @ W, rtol=0, atol=1e-11)
    np.testing.assert_allclose(dW, dY.T @ X, rtol=0, atol=1e-11)


def test_gemm_views_and_accumulate():
    """Leading dimensions and += are honoured (slices of a larger matrix)."""
    rng = np.random.default_rng(11)
    A = rng.standard_normal((9, 20))
    B = rng.standard_normal((11, 20))
    C = rng.standard_normal((9, 30))
    C0 = C.copy()
    orc.gemm_nt(A[:, 3:13], B[:, 5:15], C[:, 7:18], accumulate=True)
    np.testing.assert_allclose(C[:, 7:18], C0[:, 7:18] + A[:, 3:13] @ B[:, 5:15].T, atol=1e-12)
    assert np.array_equal(C[:, :7], C0[:, :7]) and np.array_equal(C[:, 18:], C0[:, 18:])
    D = rng.standard_normal((20, 6))
    E = np.full((9, 10), 5.0)
    orc.gemm_nn(A, D, E[:, 2:8])
    np.testing.assert_allclose(E[:, 2:8], A @ D, atol=1e-12)
    assert np.all(E[:, :2] == 5.0) and np.all(E[:, 8:] == 5.0)
    F = np.zeros((20, 6))
    orc.gemm_tn(A, C0[:, :6], F)
    np.testing.assert_allclose(F, A.T @ C0[:, :6], atol=1e-12)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 6, 12])
def test_rotated_equals_plain_bit_for_bit(n):
    """Output partition + concat is the unsharded product; each output element
    is the same sequential sum, so equality is exact in fp64."""
    X, W, dY = rng_mats(n, 5, 7, 12)
    Yp = orc.plain_linear_fwd(X, W)
    dXp, dWp = orc.plain_linear_bwd(X, W, dY)
    for r in range(n):
        res = orc.rtp_linear_out(X, W, dY, n, r)
        assert np.array_equal(res["Y"], Yp)
        assert np.array_equal(res["G"], dWp)
        np.testing.assert_allclose(res["dX"], dXp, rtol=0, atol=1e-12)   # order of the sum over shards differs
        assert np.array_equal(res["W_after"], W), "every shard returns unchanged"
        assert res["fwd_log"] == [(t, (r - t) % n) for t in range(n)]
        assert res["bwd_log"] == [(s, (r + 1 + s) % n) for s in range(n)]
        assert res["resident_after_fwd"] == (r + 1) % n
        assert res["resident_after_bwd"] == r
        assert res["fwd_rotations"] == n - 1 and res["bwd_rotations"] == n - 1
        # each shard is sent and received at most once per pass by this worker
        assert len(set(res["sent"][:n - 1])) == n - 1 and len(set(res["received"][:n - 1])) == n - 1


@pytest.mark.parametrize("n", [1, 2, 3, 4, 6])
def test_input_partition_sums_to_plain(n):
    """Input-dimension partition: the N partial products add up to the full one."""
    rng = np.random.default_rng(5)
    T, I, O = 4, 12, 7
    X, W, dY = rng.standard_normal((T, I)), rng.standard_normal((O, I)), rng.standard_normal((T, O))
    for r in range(n):
        res = orc.rtp_linear_in(X, W, dY, n, r)
        np.testing.assert_allclose(res["Y"], X @ W.T, rtol=0, atol=1e-12)
        np.testing.assert_allclose(res["dX"], dY @ W, rtol=0, atol=1e-12)
        np.testing.assert_allclose(res["G"], dY.T @ X, rtol=0, atol=1e-12)
        assert np.array_equal(res["W_after"], W)
        assert res["resident_after_bwd"] == r


def test_gradient_accumulates_onto_arriving_content():
    X, W, dY = rng_mats(9, 6, 5, 8)
    G0 = np.random.default_rng(10).standard_normal(W.shape)
    res = orc.rtp_linear_out(X, W, dY, 4, 2, G0=G0)
    np.testing.assert_allclose(res["G"], G0 + dY.T @ X, rtol=0, atol=1e-12)
    res = orc.rtp_linear_in(X, W, dY, 1, 0, G0=G0)
    np.testing.assert_allclose(res["G"], G0 + dY.T @ X, rtol=0, atol=1e-12)
    Xw = np.random.default_rng(12).standard_normal((6, 8))
    Ww = np.random.default_rng(13).standard_normal((5, 8))
    G0w = np.random.default_rng(14).standard_normal((5, 8))
    res = orc.rtp_linear_in(Xw, Ww, dY[:, :5], 4, 3, G0=G0w)
    np.testing.assert_allclose(res["G"], G0w + dY[:, :5].T @ Xw, rtol=0, atol=1e-12)


def test_structured_cases():
    rng = np.random.default_rng(21)
    I = 6
    W = rng.standard_normal((8, I))
    # X = identity  =>  Y = W^T
    res = orc.rtp_linear_out(np.eye(I), W, np.zeros((I, 8)), 4, 0)
    assert np.array_equal(res["Y"], W.T)
    # dY = 0  =>  gradients untouched, dX = 0
    assert np.array_equal(res["G"], np.zeros_like(W)) and np.array_equal(res["dX"], np.zeros((I, I)))
    # one-hot rows of W  =>  Y gathers columns of X
    X = rng.standard_normal((5, I))
    sel = [3, 0, 5, 1, 1, 2, 4, 0]
    W1h = np.zeros((8, I))
    W1h[np.arange(8), sel] = 1.0
    res = orc.rtp_linear_out(X, W1h, np.zeros((5, 8)), 8, 3)   # n == O: one column per step
    assert np.array_equal(res["Y"], X[:, sel])
    # n == 1 is the plain linear
    dY = rng.standard_normal((5, 8))
    res = orc.rtp_linear_out(X, W, dY, 1, 0)
    assert np.array_equal(res["Y"], orc.plain_linear_fwd(X, W))


@pytest.mark.parametrize("n", [2, 3, 4])
def test_full_ring_reduces_gradients(n):
    """All N workers: the concat of their outputs is the global product and the
    gradient shard that arrives back at its owner is the sum over all workers,
    so no separate all-reduce is needed; everybody sends and receives each
    shard at most once per pass."""
    rng = np.random.default_rng(n)
    Tg, I, O = 2 * n, 5, 3 * n
    X, W, dY = rng.standard_normal((Tg, I)), rng.standard_normal((O, I)), rng.standard_normal((Tg, O))
    res = orc.ring_linear_out(X, W, dY, n)
    np.testing.assert_allclose(res["Y"], X @ W.T, rtol=0, atol=1e-12)
    np.testing.assert_allclose(res["dX"], dY @ W, rtol=0, atol=1e-12)
    np.testing.assert_allclose(res["dW"], dY.T @ X, rtol=0, atol=1e-12)
    assert np.array_equal(res["W_after"], W)
    for r in range(n):
        assert len(res["sends"][r]) == 2 * (n - 1) and len(res["recvs"][r]) == 2 * (n - 1)
        assert len(set(res["sends"][r][:n - 1])) == n - 1 and len(set(res["sends"][r][n - 1:])) == n - 1
    assert len(res["history"]) == 2 * n


# --------------------------------------------------------------- activations --

def test_activation_closed_forms():
    from scipy.special import ndtr, expit
    x = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(orc.act(x, orc.GELU_ERF), x * ndtr(x), rtol=0, atol=1e-15)
    np.testing.assert_allclose(orc.act(x, orc.SILU), x * expit(x), rtol=0, atol=1e-15)
    assert orc.act(np.array([0.0]), orc.GELU_ERF)[0] == 0.0
    assert orc.act_grad(np.array([0.0]), orc.GELU_ERF)[0] == 0.5
    assert orc.act_grad(np.array([0.0]), orc.SILU)[0] == 0.5
    assert orc.act_grad(np.array([0.0]), orc.GELU_TANH)[0] == 0.5
    # far tails: identity on the right, zero on the left
    np.testing.assert_allclose(orc.act(np.array([30.0, -30.0]), orc.GELU_ERF), [30.0, 0.0], atol=1e-15)
    np.testing.assert_allclose(orc.act(np.array([40.0, -40.0]), orc.SILU), [40.0, 0.0], atol=1e-15)
    # the tanh form approximates the erf form to about 1e-3 (known property)
    assert np.abs(orc.act(x, orc.GELU_TANH) - orc.act(x, orc.GELU_ERF)).max() < 2e-3


def test_tanh_gelu_value_and_derivative_against_a_library_routine():
    """The tanh form pinned to rounding error: a library's own implementation of it in fp64 (value, and the
    derivative through that library's automatic differentiation), the odd-part identity g(x) - g(-x) = x that
    follows from tanh being odd, and the tails."""
    import torch
    x = np.linspace(-8, 8, 641)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.gelu(xt, approximate="tanh")
    yt.sum().backward()
    np.testing.assert_allclose(orc.act(x, orc.GELU_TANH), yt.detach().numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(orc.act_grad(x, orc.GELU_TANH), xt.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(orc.act(x, orc.GELU_TANH) - orc.act(-x, orc.GELU_TANH), x, rtol=0, atol=1e-14)
    np.testing.assert_allclose(orc.act(np.array([30.0, -30.0]), orc.GELU_TANH), [30.0, 0.0], atol=1e-15)


@pytest.mark.parametrize("kind", [orc.GELU_ERF, orc.GELU_TANH, orc.SILU])
def test_activation_derivative_by_central_difference(kind):
    x = np.linspace(-5, 5, 101)
    h = 1e-5
    fd = (orc.act(x + h, kind) - orc.act(x - h, kind)) / (2 * h)
    np.testing.assert_allclose(orc.act_grad(x, kind), fd, rtol=0, atol=1e-9)


# --------------------------------------------------- composites and gradients --

def _fd_check(loss_fn, params, grads, eps=1e-6, samples=12, seed=0, tol=2e-7):
    rng = np.random.default_rng(seed)
    for name, P in params.items():
        for _ in range(samples):
            idx = tuple(rng.integers(0, s) for s in P.shape)
            old = P[idx]
            P[idx] = old + eps
            lp = loss_fn()
            P[idx] = old - eps
            lm = loss_fn()
            P[idx] = old
            fd = (lp - lm) / (2 * eps)
            g = grads[name][idx]
            assert abs(fd - g) <= tol * max(1.0, abs(g)), (name, idx, fd, g)


def test_linear_gradients_by_finite_differences():
    """L = sum(Y * dY)  =>  dL/dX = dY W and dL/dW = dY^T X."""
    X, W, dY = rng_mats(31, 4, 5, 6)
    res = orc.rtp_linear_out(X, W, dY, 3, 1)
    _fd_check(lambda: float(np.sum(orc.plain_linear_fwd(X, W) * dY)), {"X": X, "W": W},
              {"X": res["dX"], "W": res["G"]})


@pytest.mark.parametrize("kind", [orc.GELU_ERF, orc.GELU_TANH])
def test_mlp_rotated_matches_plain_and_fd(kind):
    rng = np.random.default_rng(41)
    T, I, O1, O2, n = 4, 5, 12, 3, 4
    X, W1, W2 = rng.standard_normal((T, I)), rng.standard_normal((O1, I)) * 0.5, rng.standard_normal((O2, O1)) * 0.5
    dY = rng.standard_normal((T, O2))
    plain = orc.plain_mlp(X, W1, W2, dY, kind)
    for r in range(n):
        rot = orc.rtp_mlp(X, W1, W2, dY, n, r, kind)
        for a, b in (("Y", "Y"), ("dX", "dX"), ("dW1", "dW1"), ("dW2", "dW2"), ("Z", "Z"), ("H", "H")):
            np.testing.assert_allclose(rot[a], plain[b], rtol=0, atol=1e-12)
        assert rot["resident_after_bwd"] == r
    _fd_check(lambda: float(np.sum(orc.plain_mlp(X, W1, W2, dY, kind)["Y"] * dY)),
              {"X": X, "W1": W1, "W2": W2}, {"X": plain["dX"], "W1": plain["dW1"], "W2": plain["dW2"]})


def test_swiglu_rotated_matches_plain_and_fd():
    rng = np.random.default_rng(43)
    T, I, O1, O2, n = 3, 4, 6, 5, 3
    X = rng.standard_normal((T, I))
    Wg, Wu = rng.standard_normal((O1, I)) * 0.7, rng.standard_normal((O1, I)) * 0.7
    Wd = rng.standard_normal((O2, O1)) * 0.7
    dY = rng.standard_normal((T, O2))
    plain = orc.plain_swiglu(X, Wg, Wu, Wd, dY)
    # the forward against a separate statement with library routines
    from scipy.special import expit
    A, B = X @ Wg.T, X @ Wu.T
    np.testing.assert_allclose(plain["Y"], (A * expit(A) * B) @ Wd.T, rtol=0, atol=1e-12)
    for r in range(n):
        rot = orc.rtp_swiglu(X, Wg, Wu, Wd, dY, n, r)
        for key in ("Y", "dX", "dWg", "dWu", "dWd", "A", "B", "H"):
            np.testing.assert_allclose(rot[key], plain[key], rtol=0, atol=1e-12)
    _fd_check(lambda: float(np.sum(orc.plain_swiglu(X, Wg, Wu, Wd, dY)["Y"] * dY)),
              {"X": X, "Wg": Wg, "Wu": Wu, "Wd": Wd},
              {"X": plain["dX"], "Wg": plain["dWg"], "Wu": plain["dWu"], "Wd": plain["dWd"]})


def test_composites_accumulate_onto_arriving_gradients():
    rng = np.random.default_rng(47)
    T, I, O1, O2, n = 3, 4, 6, 5, 3
    X = rng.standard_normal((T, I))
    Wg, Wu, Wd = rng.standard_normal((O1, I)), rng.standard_normal((O1, I)), rng.standard_normal((O2, O1))
    dY = rng.standard_normal((T, O2))
    G = [rng.standard_normal(w.shape) for w in (Wg, Wu, Wd)]
    base = orc.rtp_swiglu(X, Wg, Wu, Wd, dY, n, 1)
    withg = orc.rtp_swiglu(X, Wg, Wu, Wd, dY, n, 1, *G)
    for key, g in zip(("dWg", "dWu", "dWd"), G):
        np.testing.assert_allclose(withg[key], base[key] + g, rtol=0, atol=1e-12)


# ------------------------------------------------------------------ Table 1 --

def _table1():
    rows = {}
    with open(os.path.join(GOLDEN, "table1_param_memory.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, cost, dup = [c.strip() for c in line.split("|")]
            rows[name] = (cost, dup)
    return rows


@pytest.mark.parametrize("W,G,N", [(100, 100, 4), (939524096, 1879048192, 16), (64, 32, 8), (7, 9, 2)])
def test_table1_closed_forms(W, G, N):
    for name, (cost, dup) in _table1().items():
        env = {"W": W, "G": G, "N": N, "max": max}
        assert orc.param_bytes(name, W, G, N) == eval(cost, env), name
        if name not in ("tensor_parallel", "pipeline_parallel"):
            assert orc.param_duplication(name, W, G, N) == eval(dup, env), name


def test_table1_large_config_numbers():
    """The large single-worker-share config: up [28672, 8192] and down
    [8192, 28672] in bf16 with fp32 gradient shards over 16 workers."""
    elems = 2 * 28672 * 8192
    W, G, N = elems * 2, elems * 4, 16
    assert W == 939_524_096 and G == 1_879_048_192
    assert orc.param_bytes("rtp", W, G, N) == 4_697_620_480
    assert orc.worker_param_bytes("rtp", W, G, N) == 293_601_280
    assert orc.worker_param_bytes("rtp_inplace", W, G, N) == 176_160_768
    assert orc.worker_param_bytes("rtp", W, W, N) == 176_160_768     # bf16 gradient shards


# ------------------------------------------------------------------ bias in the flat parameter --

def test_bias_plain_vs_brute_force():
    """Y[t, j] = sum_i X[t, i] W[j, i] + b[j] and db[j] = sum_t dY[t, j], written out element by element
    in extended precision."""
    T, I, O = 5, 4, 6
    X, W, dY = rng_mats(91, T, I, O)
    b = np.random.default_rng(92).standard_normal(O)
    Yb = np.zeros((T, O), dtype=np.longdouble)
    db = np.zeros(O, dtype=np.longdouble)
    for t in range(T):
        for j in range(O):
            acc = np.longdouble(b[j])
            for i in range(I):
                acc += np.longdouble(X[t, i]) * np.longdouble(W[j, i])
            Yb[t, j] = acc
            db[j] += np.longdouble(dY[t, j])
    np.testing.assert_allclose(orc.plain_linear_fwd(X, W, b), Yb.astype(np.float64), rtol=0, atol=1e-13)
    np.testing.assert_allclose(orc.plain_bias_grad(dY), db.astype(np.float64), rtol=0, atol=1e-13)
    np.testing.assert_allclose(orc.plain_bias_grad(dY), dY.sum(axis=0), rtol=0, atol=1e-12)   # library routine


@pytest.mark.parametrize("n", [1, 2, 3, 6])
def test_bias_rides_with_its_rows(n):
    """The rotated layer with the bias carried in the shard gives the plain layer with bias, the bias
    gradient adds onto what arrives with the shard, and weights and bias come back unchanged."""
    T, I, O = 7, 5, 12
    X, W, dY = rng_mats(93 + n, T, I, O)
    rng = np.random.default_rng(94)
    b, gb0, G0 = rng.standard_normal(O), rng.standard_normal(O), rng.standard_normal((O, I))
    for rank in range(n):
        res = orc.rtp_linear_out_bias(X, W, b, dY, n, rank, G0, gb0)
        np.testing.assert_allclose(res["Y"], orc.plain_linear_fwd(X, W, b), rtol=0, atol=1e-12)
        dX, dW = orc.plain_linear_bwd(X, W, dY)
        np.testing.assert_allclose(res["dX"], dX, rtol=0, atol=1e-12)
        np.testing.assert_allclose(res["G"], G0 + dW, rtol=0, atol=1e-12)
        np.testing.assert_allclose(res["gb"], gb0 + orc.plain_bias_grad(dY), rtol=0, atol=1e-12)
        assert np.array_equal(res["W_after"], W) and np.array_equal(res["b_after"], b)
        assert res["resident_after_bwd"] == rank


def test_bias_gradient_by_finite_differences():
    """L = sum(Y * dY) with Y = X W^T + b  =>  dL/db = column sums of dY (and dL/dX, dL/dW unchanged)."""
    X, W, dY = rng_mats(95, 4, 5, 6)
    b = np.random.default_rng(96).standard_normal(6)
    res = orc.rtp_linear_out_bias(X, W, b, dY, 3, 2)
    _fd_check(lambda: float(np.sum(orc.plain_linear_fwd(X, W, b) * dY)), {"X": X, "W": W, "b": b},
              {"X": res["dX"], "W": res["G"], "b": res["gb"]})


# ------------------------------------------------------ expert partition --

def _experts(rng, n, I, O, O2, gated, scale=0.5):
    k = 3 if gated else 2
    shapes = [(O, I), (O, I), (O2, O)] if gated else [(O, I), (O2, O)]
    return [tuple(scale * rng.standard_normal(shapes[j]) for j in range(k)) for _ in range(n)]


def _numpy_expert(x, ex, gated):
    """Independent of the oracle's C routines: numpy matmul, scipy erf."""
    from scipy.special import erf
    if gated:
        Wg, Wu, Wd = ex
        a, b = Wg @ x, Wu @ x
        return Wd @ (a / (1.0 + np.exp(-a)) * b)
    W1, W2 = ex
    z = W1 @ x
    return W2 @ (0.5 * z * (1.0 + erf(z / np.sqrt(2.0))))


@pytest.mark.parametrize("align", [1, 4, 32])
def test_moe_dispatch_against_a_stable_sort(align):
    rng = np.random.default_rng(11)
    for n, T in ((1, 5), (4, 0), (4, 37), (7, 200), (16, 64)):
        route = rng.integers(0, n, T)
        if T > 10:
            route[route == n - 1] = 0                # an expert nobody is routed to
        counts, begin, perm = orc.moe_dispatch(route, n, align)
        assert counts == [int((route == e).sum()) for e in range(n)]
        order = np.argsort(route, kind="stable")     # library routine: tokens by expert, order kept
        got = [p for p in perm if p >= 0]
        assert got == list(order)
        assert len(perm) == begin[n] and all(b % align == 0 for b in begin)
        for e in range(n):
            seg = perm[begin[e]:begin[e + 1]]
            assert len(seg) < counts[e] + align
            assert all(p >= 0 for p in seg[:counts[e]]) and all(p == -1 for p in seg[counts[e]:])
            assert all(route[p] == e for p in seg[:counts[e]])


@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("n", [1, 2, 5])
def test_moe_rotated_matches_the_token_by_token_definition(n, gated):
    """Expert rotation reaches what the definition gives: every token through its own expert, every
    expert's gradient summed over its tokens onto what arrived, whatever worker does it; the
    forward output also against plain numpy."""
    rng = np.random.default_rng(100 + n)
    T, I, O, O2 = 23, 6, 5, 4
    X, dY = rng.standard_normal((T, I)), rng.standard_normal((T, O2))
    ex = _experts(rng, n, I, O, O2, gated)
    G0 = [tuple(rng.standard_normal(w.shape) for w in e) for e in ex]
    route = rng.integers(0, n, T)
    ref = orc.plain_moe(X, route, ex, dY, G0=G0)
    for t in range(T):
        np.testing.assert_allclose(ref["Y"][t], _numpy_expert(X[t], ex[route[t]], gated), rtol=1e-12, atol=1e-12)
    for rank in range(n):
        out = orc.rtp_moe(X, route, ex, dY, n, rank, G0=G0)
        np.testing.assert_allclose(out["Y"], ref["Y"], rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(out["dX"], ref["dX"], rtol=1e-13, atol=1e-13)
        for e in range(n):
            for j in range(len(ex[e])):
                np.testing.assert_allclose(out["G"][e][j], ref["G"][e][j], rtol=1e-12, atol=1e-12)
        assert [e for (_, e, _) in out["fwd_log"]] == [orc.fwd_shard(rank, t, n) for t in range(n)]
        assert [e for (_, e, _) in out["bwd_log"]] == [orc.bwd_shard(rank, s, n) for s in range(n)]
        assert out["resident_after_bwd"] == rank
        assert sum(c for (_, _, c) in out["fwd_log"]) == T, "every token is computed exactly once"


def test_moe_special_cases():
    """All tokens on one expert: that expert's plain MLP, the other experts' gradients pass through
    untouched.  Reordering the tokens reorders the outputs and leaves the weight gradients alone."""
    rng = np.random.default_rng(7)
    n, T, I, O, O2 = 4, 17, 5, 6, 3
    X, dY = rng.standard_normal((T, I)), rng.standard_normal((T, O2))
    ex = _experts(rng, n, I, O, O2, False)
    G0 = [tuple(rng.standard_normal(w.shape) for w in e) for e in ex]
    out = orc.rtp_moe(X, np.full(T, 2), ex, dY, n, 1, G0=G0)
    ref = orc.plain_mlp(X, ex[2][0], ex[2][1], dY)
    np.testing.assert_allclose(out["Y"], ref["Y"], rtol=1e-13)
    np.testing.assert_allclose(out["dX"], ref["dX"], rtol=1e-13)
    np.testing.assert_allclose(out["G"][2][0], G0[2][0] + ref["dW1"], rtol=1e-12)
    np.testing.assert_allclose(out["G"][2][1], G0[2][1] + ref["dW2"], rtol=1e-12)
    for e in (0, 1, 3):
        for j in range(2):
            assert np.array_equal(out["G"][e][j], G0[e][j])
    route = rng.integers(0, n, T)
    a = orc.rtp_moe(X, route, ex, dY, n, 0)
    sh = rng.permutation(T)
    b = orc.rtp_moe(X[sh], route[sh], ex, dY[sh], n, 0)
    np.testing.assert_allclose(b["Y"], a["Y"][sh], rtol=1e-13)
    np.testing.assert_allclose(b["dX"], a["dX"][sh], rtol=1e-13)
    for e in range(n):
        for j in range(2):
            np.testing.assert_allclose(b["G"][e][j], a["G"][e][j], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("gated", [False, True])
def test_moe_gradients_by_finite_differences(gated):
    """d/dθ of L = sum(Y * dY), with the forward taken from plain numpy, against the oracle's backward."""
    rng = np.random.default_rng(21)
    n, T, I, O, O2 = 3, 9, 4, 5, 3
    X, dY = rng.standard_normal((T, I)), rng.standard_normal((T, O2))
    ex = _experts(rng, n, I, O, O2, gated)
    route = rng.integers(0, n, T)
    out = orc.rtp_moe(X, route, ex, dY, n, 2)

    def loss(Xv, exv):
        return sum(float(_numpy_expert(Xv[t], exv[route[t]], gated) @ dY[t]) for t in range(T))

    h = 1e-6
    for (t, i) in ((0, 0), (4, 3), (8, 1)):
        Xp, Xm = X.copy(), X.copy()
        Xp[t, i] += h
        Xm[t, i] -= h
        assert abs((loss(Xp, ex) - loss(Xm, ex)) / (2 * h) - out["dX"][t, i]) < 1e-6
    for e in range(n):
        for j in range(len(ex[e])):
            r, c = rng.integers(0, ex[e][j].shape[0]), rng.integers(0, ex[e][j].shape[1])
            exp_, exm = [list(map(np.copy, x)) for x in ex], [list(map(np.copy, x)) for x in ex]
            exp_[e][j][r, c] += h
            exm[e][j][r, c] -= h
            fd = (loss(X, exp_) - loss(X, exm)) / (2 * h)
            assert abs(fd - out["G"][e][j][r, c]) < 1e-6, (e, j)


# ------------------------------------ bias of the input-partitioned layer --

@pytest.mark.parametrize("n,O", [(1, 7), (3, 7), (4, 8), (8, 5)])
def test_input_partition_bias_spread_over_the_shards(n, O):
    """Pieces of b ride with the shards (the last ones short or empty when N does not divide, or
    exceeds, the output width): the sum over the steps is X W^T + b, the pieces' gradients are the
    column sums of dY on top of what arrived, from every rank; numpy is the reference."""
    rng = np.random.default_rng(40 + n)
    T, I = 6, 4 * n
    X, W, dY = rng.standard_normal((T, I)), rng.standard_normal((O, I)), rng.standard_normal((T, O))
    b, gb0, G0 = rng.standard_normal(O), rng.standard_normal(O), rng.standard_normal((O, I))
    pieces = orc.bias_pieces(O, n)
    assert pieces[0][0] == 0 and pieces[-1][1] == O and all(a[1] == c[0] for a, c in zip(pieces, pieces[1:]))
    sizes = [hi - lo for lo, hi in pieces]
    assert sum(sizes) == O and max(sizes) == -(-O // n) and sizes == sorted(sizes, reverse=True)
    for rank in range(n):
        out = orc.rtp_linear_in(X, W, dY, n, rank, G0=G0, b=b, gb0=gb0)
        np.testing.assert_allclose(out["Y"], X @ W.T + b[None, :], rtol=0, atol=1e-12)
        np.testing.assert_allclose(out["gb"], gb0 + dY.sum(axis=0), rtol=0, atol=1e-12)
        np.testing.assert_allclose(out["G"], G0 + dY.T @ X, rtol=0, atol=1e-12)
        np.testing.assert_allclose(out["dX"], dY @ W, rtol=0, atol=1e-12)
        assert np.array_equal(out["b_after"], b) and np.array_equal(out["W_after"], W)
    # W = 0: the output is the bias on every row
    out = orc.rtp_linear_in(X, np.zeros_like(W), dY, n, 0, b=b)
    assert np.array_equal(out["Y"], np.tile(b, (T, 1)))


@pytest.mark.parametrize("kind", [orc.GELU_ERF, orc.GELU_TANH])
def test_mlp_with_biases_rotated_matches_plain_numpy_and_fd(kind):
    from scipy.special import erf
    rng = np.random.default_rng(77)
    n, T, I, O1, O2 = 4, 5, 6, 8, 7
    X, dY = rng.standard_normal((T, I)), rng.standard_normal((T, O2))
    W1, W2 = 0.5 * rng.standard_normal((O1, I)), 0.5 * rng.standard_normal((O2, O1))
    b1, b2 = rng.standard_normal(O1), rng.standard_normal(O2)
    gb1_0, gb2_0 = rng.standard_normal(O1), rng.standard_normal(O2)
    ref = orc.plain_mlp(X, W1, W2, dY, kind, b1=b1, b2=b2)
    if kind == orc.GELU_ERF:
        z = X @ W1.T + b1
        np.testing.assert_allclose(ref["Y"], (0.5 * z * (1 + erf(z / np.sqrt(2)))) @ W2.T + b2, rtol=1e-12, atol=1e-12)
    for rank in (0, 3):
        out = orc.rtp_mlp(X, W1, W2, dY, n, rank, kind, b1=b1, b2=b2, gb1_0=gb1_0, gb2_0=gb2_0)
        for key in ("Y", "dX", "dW1", "dW2"):
            np.testing.assert_allclose(out[key], ref[key], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(out["db1"], gb1_0 + ref["db1"], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(out["db2"], gb2_0 + ref["db2"], rtol=1e-12, atol=1e-12)
    # finite differences of L = sum(Y * dY) in the two biases
    out = orc.rtp_mlp(X, W1, W2, dY, n, 1, kind, b1=b1, b2=b2)
    h = 1e-6
    loss = lambda c1, c2: float((orc.plain_mlp(X, W1, W2, dY, kind, b1=c1, b2=c2)["Y"] * dY).sum())
    for j in (0, 5):
        e1, e2 = np.zeros(O1), np.zeros(O2)
        e1[j], e2[j] = h, h
        assert abs((loss(b1 + e1, b2) - loss(b1 - e1, b2)) / (2 * h) - out["db1"][j]) < 1e-6
        assert abs((loss(b1, b2 + e2) - loss(b1, b2 - e2)) / (2 * h) - out["db2"][j]) < 1e-6


def test_gated_unit_with_biases_rotated_matches_plain_numpy_and_fd():
    """Biases of the gated unit: the unsharded definition against a numpy forward and central differences in
    every bias, and the rotated form against the unsharded one (arriving bias gradients added onto)."""
    from scipy.special import expit
    rng = np.random.default_rng(91)
    n, T, I, O1, O2 = 4, 5, 6, 8, 7
    X, dY = rng.standard_normal((T, I)), rng.standard_normal((T, O2))
    Wg, Wu, Wd = 0.5 * rng.standard_normal((O1, I)), 0.5 * rng.standard_normal((O1, I)), 0.5 * rng.standard_normal((O2, O1))
    bg, bu, bd = rng.standard_normal(O1), rng.standard_normal(O1), rng.standard_normal(O2)
    g0 = [rng.standard_normal(O1), rng.standard_normal(O1), rng.standard_normal(O2)]
    ref = orc.plain_swiglu(X, Wg, Wu, Wd, dY, bg, bu, bd)
    a, b = X @ Wg.T + bg, X @ Wu.T + bu
    np.testing.assert_allclose(ref["Y"], (a * expit(a) * b) @ Wd.T + bd, rtol=1e-12, atol=1e-12)
    nobias = orc.plain_swiglu(X, Wg, Wu, Wd, dY)
    zero = orc.plain_swiglu(X, Wg, Wu, Wd, dY, np.zeros(O1), np.zeros(O1), np.zeros(O2))
    for key in ("Y", "dX", "dWg", "dWu", "dWd"):
        assert np.array_equal(nobias[key], zero[key]), "zero biases change nothing"
    for rank in (0, 3):
        out = orc.rtp_swiglu(X, Wg, Wu, Wd, dY, n, rank, bg=bg, bu=bu, bd=bd, gbg0=g0[0], gbu0=g0[1], gbd0=g0[2])
        for key in ("Y", "dX", "dWg", "dWu", "dWd"):
            np.testing.assert_allclose(out[key], ref[key], rtol=1e-12, atol=1e-12)
        for key, arriving in zip(("dbg", "dbu", "dbd"), g0):
            np.testing.assert_allclose(out[key], arriving + ref[key], rtol=1e-12, atol=1e-12)
    h = 1e-6
    loss = lambda cg, cu, cd: float((orc.plain_swiglu(X, Wg, Wu, Wd, dY, cg, cu, cd)["Y"] * dY).sum())
    for j in (0, 5):
        e1, e2 = np.zeros(O1), np.zeros(O2)
        e1[j], e2[j] = h, h
        assert abs((loss(bg + e1, bu, bd) - loss(bg - e1, bu, bd)) / (2 * h) - ref["dbg"][j]) < 1e-6
        assert abs((loss(bg, bu + e1, bd) - loss(bg, bu - e1, bd)) / (2 * h) - ref["dbu"][j]) < 1e-6
        assert abs((loss(bg, bu, bd + e2) - loss(bg, bu, bd - e2)) / (2 * h) - ref["dbd"][j]) < 1e-6
