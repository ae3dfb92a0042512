"""Pins of the oracle's layer-wise reconstruction step (Alg. 1, Sec. 4.2) against what the paper and
the mathematics fix.  CPU only.  Nothing here calls the HIP path.

The oracle differentiates the forward pass of Alg. 1 as written (Z, Z', the sum of squares, back
through B.A.X^T).  The pins reach the same numbers by other routes:
  * the loss through the trace form tr(Delta_F X^T X Delta_F^T) of Sec. 4.2;
  * the gradients through the closed form dL/dSigma = -2 Delta_F X^T X of Sec. 4.2 and the chain
    rule through Sigma = B.A;
  * central differences of the loss with Q(W - Sigma) held fixed (the "detached" graph);
  * the exact zero of dL/dA while B = 0 (Alg. 1 initialises B with zeros), the identity quantizer
    (straight-through: Delta_F vanishes identically, so does the gradient), a triple loop on a tiny
    layer, the s/2 bound of Sec. 4.1 after every update, and descent of the detached loss.
"""
import numpy as np
import pytest

import fbq_synth
from oracle import fbq_oracle as orc


def _problem(N, K, r, bits, T, seed, b_zero=False, group=128):
    spec = fbq_synth.LayerSpec("train", N, K, r, bits, group)
    W = fbq_synth.make_weight(spec, 31, seed)
    A16, B16 = fbq_synth.make_branch(spec, 31, seed)
    X = fbq_synth.make_x(spec, T, 31, seed)
    A = A16.astype(np.float64)
    B = np.zeros((r, N)) if b_zero else B16.astype(np.float64)
    return spec, W, X, np.ascontiguousarray(A), np.ascontiguousarray(B)


def _wq(out, group):
    s = np.repeat(out["scales"].astype(np.float64), group, axis=1)
    z = np.repeat(out["zeros"].astype(np.float64), group, axis=1)
    return s * (out["codes"].astype(np.float64) - z)


def _detached_loss(W, X, Wq, A, B):
    """|| W X^T - (Wq X^T + (A B)^T X^T) ||_F^2 with the quantized weight a constant."""
    Xd = X.astype(np.float64)
    Zdiff = (W.astype(np.float64) - Wq - (A @ B).T) @ Xd.T
    return float(np.sum(Zdiff * Zdiff))


@pytest.mark.parametrize("bits", [4, 3])
def test_loss_equals_trace_form(bits):
    spec, W, X, A, B = _problem(48, 256, 8, bits, 40, 1)
    out = orc.train_step(W, X, A.copy(), B.copy(), 0.0, bits, spec.group)
    Sigma = (out["A16"].astype(np.float64) @ out["B16"].astype(np.float64)).T
    Delta = W.astype(np.float64) - _wq(out, spec.group) - Sigma          # Delta_F of Sec. 4.2
    H = orc.gram(X)
    trace = float(np.trace(Delta @ H @ Delta.T))
    assert out["loss"] == pytest.approx(trace, rel=1e-10)


@pytest.mark.parametrize("bits", [4, 3])
def test_gradients_equal_closed_form(bits):
    spec, W, X, A, B = _problem(64, 256, 16, bits, 50, 2)
    out = orc.train_step(W, X, A.copy(), B.copy(), 0.0, bits, spec.group)
    A16, B16 = out["A16"].astype(np.float64), out["B16"].astype(np.float64)
    Delta = W.astype(np.float64) - _wq(out, spec.group) - (A16 @ B16).T
    gSigma = -2.0 * Delta @ orc.gram(X)                                  # [N,K], Sec. 4.2
    # Sigma[n,k] = sum_j A[k,j] B[j,n]
    gA = gSigma.T @ B16.T
    gB = A16.T @ gSigma.T
    assert np.allclose(out["gradA"], gA, rtol=1e-9, atol=1e-12 * np.abs(gA).max())
    assert np.allclose(out["gradB"], gB, rtol=1e-9, atol=1e-12 * np.abs(gB).max())


def test_gradients_equal_central_differences_of_the_detached_loss():
    spec, W, X, A, B = _problem(16, 128, 8, 4, 12, 3)
    out = orc.train_step(W, X, A.copy(), B.copy(), 0.0, 4, spec.group)
    A16, B16 = out["A16"].astype(np.float64), out["B16"].astype(np.float64)
    Wq = _wq(out, spec.group)
    rng = np.random.default_rng(5)
    h = 1e-5
    for _ in range(12):
        k, j, n = rng.integers(spec.K), rng.integers(spec.r), rng.integers(spec.N)
        Ap, Am = A16.copy(), A16.copy()
        Ap[k, j] += h
        Am[k, j] -= h
        fd = (_detached_loss(W, X, Wq, Ap, B16) - _detached_loss(W, X, Wq, Am, B16)) / (2 * h)
        assert out["gradA"][k, j] == pytest.approx(fd, rel=1e-5, abs=1e-7 * np.abs(out["gradA"]).max())
        Bp, Bm = B16.copy(), B16.copy()
        Bp[j, n] += h
        Bm[j, n] -= h
        fd = (_detached_loss(W, X, Wq, A16, Bp) - _detached_loss(W, X, Wq, A16, Bm)) / (2 * h)
        assert out["gradB"][j, n] == pytest.approx(fd, rel=1e-5, abs=1e-7 * np.abs(out["gradB"]).max())


def test_zero_B_gives_zero_gradient_for_A_and_moves_only_B():
    spec, W, X, A, B = _problem(32, 128, 8, 4, 20, 4, b_zero=True)
    A0 = A.copy()
    out = orc.train_step(W, X, A, B, 1e-4, 4, spec.group)
    assert np.all(out["gradA"] == 0.0)
    assert np.array_equal(A, A0)
    assert np.abs(out["gradB"]).max() > 0.0
    assert np.array_equal(B, -1e-4 * out["gradB"])
    # with Sigma = 0 the codes are those of plain group-wise round-to-nearest of W
    codes, s, z = orc.quantize(W, None, None, 4, spec.group)
    assert np.array_equal(out["codes"], codes) and np.array_equal(out["scales"], s) and np.array_equal(out["zeros"], z)


def test_straight_through_quantizer_gives_zero_gradient():
    """Sec. 4.2: with dQ/dW = I the two occurrences of Sigma cancel.  Written out: if the quantizer
    is replaced by the identity, Delta_F = W - (W - Sigma) - Sigma vanishes for every Sigma, so the
    loss is constant (zero) and no finite difference of it is non-zero."""
    spec, W, X, A, B = _problem(8, 128, 8, 4, 6, 5)
    Wd = W.astype(np.float64)
    for scale in (0.0, 1.0, 3.0):
        Sigma = scale * (A @ B).T
        Delta = Wd - (Wd - Sigma) - Sigma
        assert np.abs(Delta).max() <= 4 * np.finfo(np.float64).eps * np.abs(Wd).max() * max(scale, 1.0)


def test_tiny_layer_against_triple_loops():
    N, K, r, T, g = 4, 8, 8, 3, 8
    spec, W, X, A, B = _problem(N, K, r, 4, T, 6, group=g)
    out = orc.train_step(W, X, A.copy(), B.copy(), 0.0, 4, g)
    A16, B16 = out["A16"].astype(float), out["B16"].astype(float)
    Wd, Xd = W.astype(float), X.astype(float)
    loss = 0.0
    gA = [[0.0] * r for _ in range(K)]
    gB = [[0.0] * N for _ in range(r)]
    for n in range(N):
        for t in range(T):
            e = 0.0
            for k in range(K):
                wq = float(out["scales"][n, k // g]) * (float(out["codes"][n, k]) - float(out["zeros"][n, k // g]))
                sig = sum(A16[k, j] * B16[j, n] for j in range(r))
                e += (Wd[n, k] - wq - sig) * Xd[t, k]
            loss += e * e
            for j in range(r):
                gB[j][n] += -2.0 * e * sum(Xd[t, k] * A16[k, j] for k in range(K))
                for k in range(K):
                    gA[k][j] += -2.0 * e * Xd[t, k] * B16[j, n]
    assert out["loss"] == pytest.approx(loss, rel=1e-12)
    assert np.allclose(out["gradA"], np.array(gA), rtol=1e-10, atol=1e-14)
    assert np.allclose(out["gradB"], np.array(gB), rtol=1e-10, atol=1e-14)


@pytest.mark.parametrize("bits", [4, 3])
def test_bound_holds_after_every_update_and_detached_loss_descends(bits):
    spec, W, X, A, B = _problem(64, 256, 16, bits, 64, 7, b_zero=True)
    H = orc.gram(X)
    lr = 0.05 / float(np.linalg.eigvalsh(H)[-1] * max(np.linalg.norm(A, 2) ** 2, 1e-12))
    losses = []
    for step in range(6):
        A_before, B_before = A.copy(), B.copy()
        out = orc.train_step(W, X, A, B, lr, bits, spec.group)
        losses.append(out["loss"])
        # Sec. 4.1: |W - W_F| <= s/2 for the layer written by this step, whatever A and B have become
        A16, B16 = out["A16"].astype(np.float64), out["B16"].astype(np.float64)
        WF = _wq(out, spec.group) + (A16 @ B16).T
        s = np.repeat(out["scales"].astype(np.float64), spec.group, axis=1)
        assert np.all(np.abs(W.astype(np.float64) - WF) <= 0.5 * s * (1 + 1e-9))
        assert np.array_equal(out["A16"], A_before.astype(np.float16)) and np.array_equal(out["B16"], B_before.astype(np.float16))
        # the update is a descent step of the loss it differentiated (quantized weight held fixed)
        Wq = _wq(out, spec.group)
        before = _detached_loss(W, X, Wq, A16, B16)
        after = _detached_loss(W, X, Wq, A16 - lr * out["gradA"], B16 - lr * out["gradB"])
        assert after < before
        assert np.allclose(A, A_before - lr * out["gradA"], rtol=0, atol=0)
        assert np.allclose(B, B_before - lr * out["gradB"], rtol=0, atol=0)
    assert losses[-1] < losses[0]


def test_gram_is_the_plain_definition():
    spec, W, X, A, B = _problem(8, 128, 8, 4, 5, 8)
    H = orc.gram(X)
    Xd = X.astype(np.float64)
    i, j = 3, 77
    assert H[i, j] == pytest.approx(sum(Xd[t, i] * Xd[t, j] for t in range(5)), rel=1e-14)
    assert np.array_equal(H, H.T)
