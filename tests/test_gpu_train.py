"""GPU parity of the layer-wise reconstruction step (Alg. 1, Sec. 4.2) against the fp64 oracle,
through the C ABI.

Tolerances.  The quantizer runs the oracle's fp64 arithmetic, so codes, scales and zeros are compared
exactly (a code may differ on an exact tie of the rounding; none is expected on these inputs and at
most 1e-4 of the elements is accepted).  Delta_F, H and Delta_F.H enter the matrix cores rounded to
fp16 (2^-11 relative each, independent) and are accumulated in fp32: every gradient entry is a sum of
thousands of such products, so the relative L2 error of a gradient is a few 1e-4; the bar is 2e-3 for
the gradients and the updated masters' movement, 1e-3 for the loss.
"""
import numpy as np
import pytest
import torch

import fbq_synth
import paper_2501_16385_amd as fbq
from helpers import rel_l2
from oracle import fbq_oracle as orc

pytestmark = pytest.mark.gpu


def _dev16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def _problem(N, K, r, bits, T, seed, b_zero):
    spec = fbq_synth.LayerSpec("train", N, K, r, bits)
    W = fbq_synth.make_weight(spec, 33, seed)
    A16, B16 = fbq_synth.make_branch(spec, 33, seed)
    X = fbq_synth.make_x(spec, T, 33, seed)
    A = np.ascontiguousarray(A16.astype(np.float64))
    B = np.zeros((r, N)) if b_zero else np.ascontiguousarray(B16.astype(np.float64))
    return spec, W, X, A, B


@pytest.mark.parametrize("K,T", [(256, 100), (1408, 321), (256, 4100)])     # the last one: few tiles, long contraction, K split over blocks
def test_gram_matches_definition(K, T):
    spec = fbq_synth.LayerSpec("gram", 128, K, 8, 4)
    X = fbq_synth.make_x(spec, T, 33, 1)
    d = fbq.Desc(128, K, 8, 4)
    h_scale = 1.0 / T
    H16 = fbq.gram(d, _dev16(X).view(torch.float16), h_scale)
    torch.cuda.synchronize()
    want = orc.gram(X) * h_scale
    assert rel_l2(H16.cpu().numpy().astype(np.float64), want) < 5e-4


CASES = [
    # N, K, r, T, B zero at the start (Alg. 1's initialisation)
    (256, 512, 16, 200, False),
    (300, 1408, 24, 130, False),      # ragged N: partial tiles, zero padding of the transposed operands
    (384, 1024, 64, 256, True),
    (130, 256, 8, 70, False),
    (256, 512, 128, 96, False),       # rank 128: the stacked operand [Q; At] spans two tile rows
    (1100, 384, 40, 64, False),       # more rows than input features; a rank that is no multiple of 16
]


@pytest.mark.parametrize("bits", [4, 3])
@pytest.mark.parametrize("N,K,r,T,b_zero", CASES)
def test_train_step_matches_oracle(bits, N, K, r, T, b_zero):
    spec, W, X, A, B = _problem(N, K, r, bits, T, 2, b_zero)
    d = fbq.Desc(N, K, r, bits)
    Hfull = orc.gram(X)
    h_scale = 1.0 / T
    lr = 0.02 / float(np.linalg.eigvalsh(Hfull)[-1] * np.linalg.norm(A, 2) ** 2)

    At32 = torch.from_numpy(np.ascontiguousarray(A.T).astype(np.float32)).cuda()
    Bt32 = torch.from_numpy(np.ascontiguousarray(B.T).astype(np.float32)).cuda()
    # both sides start from the same masters: the fp32 values
    A = np.ascontiguousarray(At32.cpu().numpy().T.astype(np.float64))
    B = np.ascontiguousarray(Bt32.cpu().numpy().T.astype(np.float64))
    st = fbq.train_state(d, At32, Bt32)
    Wd = _dev16(W).view(torch.float16)
    H16 = fbq.gram(d, _dev16(X).view(torch.float16), h_scale)

    for step in range(3):
        print(f"step {step}: N={N} K={K} r={r} T={T} bits={bits}", flush=True)
        A_before, B_before = A.copy(), B.copy()
        want = orc.train_step(W, X, A, B, lr, bits, spec.group)
        fbq.train_step(st, Wd, H16, h_scale, lr)
        torch.cuda.synchronize()

        # the layer written by the step: fp16 branch exactly, quantizer output exactly
        assert np.array_equal(st.layer.At.cpu().numpy().view(np.float16), want["A16"].T)
        assert np.array_equal(st.layer.Bt.cpu().numpy().view(np.float16), want["B16"].T)
        codes = fbq.unpack_codes(st.layer).cpu().numpy()
        cdiff = codes.astype(np.int16) - want["codes"].astype(np.int16)
        assert np.mean(cdiff != 0) <= 1e-4 and np.all(np.abs(cdiff) <= 1)     # a near-tie of the rounding, one step at most
        assert np.mean(st.layer.scales.cpu().numpy().view(np.float16) != want["scales"]) <= 1e-4
        assert np.mean(st.layer.zeros.cpu().numpy().view(np.float16) != want["zeros"]) <= 1e-4

        assert float(st.loss.cpu()[0]) == pytest.approx(want["loss"], rel=1e-3)
        gA = st.grad_At.cpu().numpy().astype(np.float64).T
        gB = st.grad_Bt.cpu().numpy().astype(np.float64).T
        if b_zero and step == 0:
            assert np.all(gA == 0.0)
        else:
            assert rel_l2(gA, want["gradA"]) < 2e-3
        assert rel_l2(gB, want["gradB"]) < 2e-3

        # the update, measured as movement of the masters
        dA = st.At32.cpu().numpy().astype(np.float64).T - A_before
        dB = st.Bt32.cpu().numpy().astype(np.float64).T - B_before
        if np.abs(A - A_before).max() > 0:
            assert rel_l2(dA, A - A_before) < 2e-3
        assert rel_l2(dB, B - B_before) < 2e-3
        # keep both sides on the same trajectory: hand the oracle the GPU's fp32 masters
        A = np.ascontiguousarray(st.At32.cpu().numpy().T.astype(np.float64))
        B = np.ascontiguousarray(st.Bt32.cpu().numpy().T.astype(np.float64))


def test_zero_learning_rate_leaves_the_masters_and_writes_a_usable_layer():
    spec, W, X, A, B = _problem(256, 512, 16, 4, 64, 3, False)
    d = fbq.Desc(256, 512, 16, 4)
    At32 = torch.from_numpy(np.ascontiguousarray(A.T).astype(np.float32)).cuda()
    Bt32 = torch.from_numpy(np.ascontiguousarray(B.T).astype(np.float32)).cuda()
    a0, b0 = At32.clone(), Bt32.clone()
    st = fbq.train_state(d, At32, Bt32)
    H16 = fbq.gram(d, _dev16(X).view(torch.float16), 1.0 / 64)
    fbq.train_step(st, _dev16(W).view(torch.float16), H16, 1.0 / 64, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(At32, a0) and torch.equal(Bt32, b0)
    # the layer it wrote runs through the inference path and reproduces x.W_F^T
    x = fbq_synth.make_x(spec, 5, 33, 9)
    y = fbq.linear(st.layer, _dev16(x).view(torch.float16))
    torch.cuda.synchronize()
    codes, s, z = orc.quantize(W, A.astype(np.float16), B.astype(np.float16), 4, 128)
    want = orc.linear(x, orc.pack(codes, 4), s, z, A.astype(np.float16), B.astype(np.float16), 4, 128)
    assert rel_l2(y.cpu().numpy().astype(np.float64), want) < 1e-3


def test_step_without_loss_gives_the_same_gradients():
    spec, W, X, A, B = _problem(256, 512, 16, 4, 64, 4, False)
    d = fbq.Desc(256, 512, 16, 4)
    mk = lambda: (torch.from_numpy(np.ascontiguousarray(A.T).astype(np.float32)).cuda(),
                  torch.from_numpy(np.ascontiguousarray(B.T).astype(np.float32)).cuda())
    st1, st2 = fbq.train_state(d, *mk()), fbq.train_state(d, *mk())
    Wd = _dev16(W).view(torch.float16)
    H16 = fbq.gram(d, _dev16(X).view(torch.float16), 1.0 / 64)
    fbq.train_step(st1, Wd, H16, 1.0 / 64, 1e-3)
    fbq.train_step(st2, Wd, H16, 1.0 / 64, 1e-3, want_loss=False)
    torch.cuda.synchronize()
    assert torch.equal(st1.grad_At, st2.grad_At) and torch.equal(st1.grad_Bt, st2.grad_Bt)
    assert torch.equal(st1.At32, st2.At32) and torch.equal(st1.Bt32, st2.Bt32)


def test_reconstruction_loop_lowers_the_loss_and_keeps_the_bound():
    """Alg. 1 end to end on a small layer: B starts at zero, the loss of every iterate is evaluated, the
    last layer is checked against the oracle's loss for the same parameters and against the s/2 bound."""
    from paper_2501_16385_amd.reconstruction import reconstruct_layer
    N, K, r, T, bits = 256, 512, 16, 256, 4
    spec = fbq_synth.LayerSpec("loop", N, K, r, bits)
    W = fbq_synth.make_weight(spec, 34, 0)
    X = fbq_synth.make_x(spec, T, 34, 0)
    d = fbq.Desc(N, K, r, bits)
    lam = float(np.linalg.eigvalsh(orc.gram(X))[-1])
    a_std = 0.01
    # plain gradient descent on a product of two factors: the step that is stable at the start stops being so once B has
    # grown, so stay well below 1 / (lambda_max |A|^2)
    lr = 0.05 / (lam * (a_std * (np.sqrt(K) + np.sqrt(r))) ** 2)
    layer, losses = reconstruct_layer(d, _dev16(W).view(torch.float16), _dev16(X).view(torch.float16), 40, lr, a_std=a_std)
    torch.cuda.synchronize()
    vals = [l for _, l in losses]
    assert vals[-1] < 0.85 * vals[0], f"loss {vals[0]:.4g} -> {vals[-1]:.4g}"
    assert all(np.isfinite(vals))
    # the oracle's loss for the final parameters (lr = 0 leaves them alone)
    A16 = layer.At.cpu().numpy().view(np.float16).T
    B16 = layer.Bt.cpu().numpy().view(np.float16).T
    want = orc.train_step(W, X, np.ascontiguousarray(A16.astype(np.float64)), np.ascontiguousarray(B16.astype(np.float64)), 0.0,
                          bits, spec.group)
    assert vals[-1] == pytest.approx(want["loss"], rel=1e-3)
    # Sec. 4.1: the reconstructed weight of the trained layer stays within s/2 of W
    WF = fbq.reconstruct(layer).cpu().numpy().astype(np.float64)
    s = np.repeat(layer.scales.cpu().numpy().view(np.float16).astype(np.float64), 128, axis=1)
    assert np.all(np.abs(W.astype(np.float64) - WF) <= 0.5 * s * (1 + 1e-4) + 1e-7)
