"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test checks one part of oracle/fbq_oracle.c against what the paper or the
mathematics fixes: numpy's IEEE fp16 for the conversions, brute force over all
2^b candidates for the rounding, Python integers for the bit layout, exact
rational arithmetic for y on tiny layers, and the bound of Sec. 4.1
(|w - w_F| <= s/2) for the feedback reconstruction, including the negative
case in which the feedback is left out.
"""
from fractions import Fraction

import numpy as np
import pytest

import fbq_synth
from oracle import fbq_oracle as orc


def f64(a):
    return np.asarray(a, dtype=np.float16).astype(np.float64)


def tiny_layer(N, K, r, seed, w_std=0.02, ab_std=0.01, M=2):
    rng = np.random.Generator(np.random.Philox(seed))
    W = (rng.standard_normal((N, K)) * w_std).astype(np.float16)
    A = (rng.standard_normal((K, r)) * ab_std).astype(np.float16)
    B = (rng.standard_normal((r, N)) * ab_std).astype(np.float16)
    x = rng.standard_normal((M, K)).astype(np.float16)
    return W, A, B, x


# --------------------------------------------------------------------- fp16 conversions

def test_half_to_double_every_pattern_matches_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.half_to_double(bits)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_double_to_half_matches_numpy_on_values_ties_and_neighbours():
    bits = np.arange(0x7c00, dtype=np.uint16)                 # all non-negative finite fp16
    v = bits.view(np.float16).astype(np.float64)
    mids = (v[:-1] + v[1:]) / 2                               # exact ties between neighbours
    cases = [v, mids, np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf),
             np.array([65504.0, 65519.99, 65520.0, 65536.0, 1e9, 2.0 ** -25, 2.0 ** -24 * 0.5000001,
                       2.0 ** -26, 0.0, 1e-30])]
    rng = np.random.Generator(np.random.Philox(7))
    cases.append(rng.standard_normal(200000) * 10.0 ** rng.uniform(-8, 5, 200000))
    d = np.concatenate(cases)
    d = np.concatenate([d, -d])
    got = orc.double_to_half(d)
    with np.errstate(over="ignore"):
        want = d.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)


# --------------------------------------------------------------------- quantizer

@pytest.mark.parametrize("bits,N,K,group,r", [(4, 8, 8, 8, 2), (3, 8, 32, 32, 4), (4, 16, 256, 128, 8),
                                              (3, 16, 256, 128, 8), (4, 8, 8, 8, 0)])
def test_codes_in_range_and_argmin_by_brute_force(bits, N, K, group, r):
    W, A, B, _ = tiny_layer(N, K, r, seed=100 + bits + K)
    Aa, Bb = (A, B) if r else (None, None)
    codes, s, z = orc.quantize(W, Aa, Bb, bits, group)
    qmax = 2 ** bits - 1
    assert codes.dtype == np.uint8 and codes.min() >= 0 and codes.max() <= qmax
    # R = W - Sigma with numpy's matmul (independent of the oracle's loops)
    R = f64(W) - (f64(A) @ f64(B)).T if r else f64(W)
    sd = np.repeat(f64(s), group, axis=1)
    zd = np.repeat(f64(z), group, axis=1)
    cand = np.arange(qmax + 1, dtype=np.float64)
    err = np.abs(R[..., None] - sd[..., None] * (cand - zd[..., None]))      # [N,K,2^b]
    chosen = np.take_along_axis(err, codes[..., None].astype(np.int64), axis=2)[..., 0]
    best = err.min(axis=2)
    assert np.all(chosen <= best + 1e-12 * np.abs(sd))                        # ties: any arg-min is right
    # every group uses its whole range: min maps to code 0, max to code qmax (min-max quantizer)
    cg = codes.reshape(N, K // group, group)
    assert np.all(cg.min(axis=2) == 0) and np.all(cg.max(axis=2) == qmax)


def test_full_width_layer_bound_and_range():
    """Sec. 4.1: |W - W_F| <= s/2 elementwise on a layer with the benchmark's value recipe."""
    spec = fbq_synth.LayerSpec("pin", 96, 4096, 32, 4)
    L = fbq_synth.make_layer(spec, 1, config=9, layer_index=1)
    for bits in (4, 3):
        codes, s, z = orc.quantize(L["W"], L["A"], L["B"], bits, 128)
        words = orc.pack(codes, bits)
        WF = orc.reconstruct(words, s, z, L["A"], L["B"], spec.K, bits, 128)
        half_step = np.repeat(f64(s), 128, axis=1) / 2
        assert np.all(np.abs(f64(L["W"]) - WF) <= half_step * (1 + 1e-9) + 1e-18)


def test_feedback_identity_and_negative_case():
    """W - W_F = (W - Sigma) - Q(W - Sigma) (Sec. 4.1, the difference equation), and the bound fails
    when the sub-branch is NOT fed back into the quantizer (conventional W_Q + Sigma)."""
    N, K, r, g = 32, 512, 16, 128
    W, A, B, _ = tiny_layer(N, K, r, seed=5, ab_std=0.05)
    Sig = (f64(A) @ f64(B)).T
    assert np.allclose(orc.sigma(A, B), Sig, rtol=1e-13, atol=1e-18)
    for bits in (3, 4):
        codes, s, z = orc.quantize(W, A, B, bits, g)
        words = orc.pack(codes, bits)
        Wq = orc.dequant(words, s, z, K, bits, g)
        WF = orc.reconstruct(words, s, z, A, B, K, bits, g)
        R = f64(W) - Sig
        lhs = f64(W) - WF
        rhs = R - Wq
        assert np.max(np.abs(lhs - rhs)) <= 1e-15
        half = np.repeat(f64(s), g, axis=1) / 2
        assert np.all(np.abs(lhs) <= half * (1 + 1e-9))
        # negative: quantize W alone, then add Sigma afterwards
        codes0, s0, z0 = orc.quantize(W, None, None, bits, g)
        W_conv = orc.reconstruct(orc.pack(codes0, bits), s0, z0, A, B, K, bits, g)
        half0 = np.repeat(f64(s0), g, axis=1) / 2
        assert np.mean(np.abs(f64(W) - W_conv) > half0 * (1 + 1e-9)) > 0.05


def test_quantizer_edge_groups():
    """Constant groups, groups far from zero (fp16 zero-point rounding) and tiny ranges keep the bound."""
    g = 32
    rows = [np.full(g, 0.5), np.zeros(g), np.linspace(1.0, 1.01, g), np.linspace(-3.0, -2.99, g),
            np.linspace(-1e-6, 1e-6, g), np.linspace(-200.0, 300.0, g), np.linspace(100.0, 100.5, g)]
    W = np.stack(rows).astype(np.float16)
    for bits in (3, 4):
        codes, s, z = orc.quantize(W, None, None, bits, g)
        assert codes.max() <= 2 ** bits - 1
        assert np.all(f64(s) > 0) and np.all(np.isfinite(f64(z)))
        Wq = orc.dequant(orc.pack(codes, bits), s, z, g, bits, g)
        assert np.all(np.abs(f64(W) - Wq) <= f64(s) / 2 * (1 + 1e-9))
        u = Wq / f64(s) + f64(z)
        assert np.all(np.abs(u - np.rint(u)) < 1e-6)


# --------------------------------------------------------------------- packing

_INT3_SHIFT = [0, 3, 6, 9, 12, 16, 19, 22, 25, 28]     # field -> first bit, from the layout description


def layout_words_python(codes_row, bits):
    """Packed row built with Python integers straight from the layout description."""
    K = len(codes_row)
    words = [0] * (K * bits // 32)
    for k, q in enumerate(int(c) for c in codes_row):
        if bits == 4:
            words[k // 8] |= q << (4 * (k % 8))
        else:
            u, j = divmod(k, 32)
            if j < 30:
                words[3 * u + j // 10] |= q << _INT3_SHIFT[j % 10]
            else:
                hi = 15 if j == 30 else 31
                for c in range(3):
                    words[3 * u + c] |= ((q >> c) & 1) << hi
    return words


@pytest.mark.parametrize("bits", [3, 4])
def test_pack_layout_bit_by_bit_and_round_trip(bits):
    rng = np.random.Generator(np.random.Philox(11 + bits))
    qmax = 2 ** bits - 1
    N, K = 5, 160
    patterns = [rng.integers(0, qmax + 1, (N, K), dtype=np.uint8),
                (np.arange(N * K).reshape(N, K) % (qmax + 1)).astype(np.uint8)]
    patterns += [np.full((N, K), c, np.uint8) for c in range(qmax + 1)]
    for k in range(32):                                    # one-hot position: every slot of a unit
        p = np.zeros((1, 32 * 5), np.uint8)
        p[0, 32 + k] = qmax
        patterns.append(p)
    for codes in patterns:
        words = orc.pack(codes, bits)
        assert words.shape == (codes.shape[0], codes.shape[1] * bits // 32)
        for n in range(codes.shape[0]):
            assert [int(w) for w in words[n]] == layout_words_python(codes[n], bits)
        assert np.array_equal(orc.unpack(words, codes.shape[1], bits), codes)
    if bits == 4:                                          # textbook nibble packing with numpy
        codes = patterns[0].astype(np.uint32)
        want = sum(codes[:, i::8] << (4 * i) for i in range(8))
        assert np.array_equal(orc.pack(patterns[0], 4), want)
    if bits == 3:                                          # every bit of the three words is used exactly once
        ones = orc.pack(np.full((1, 32), 7, np.uint8), 3)
        assert [int(w) for w in ones[0]] == [0xFFFFFFFF] * 3


def test_pack_rejects_bad_input():
    with pytest.raises(ValueError):
        orc.pack(np.full((1, 32), 9, np.uint8), 3)         # code above qmax
    with pytest.raises(ValueError):
        orc.pack(np.zeros((1, 16), np.uint8), 3)           # not a whole 3-word unit
    with pytest.raises(ValueError):
        orc.pack(np.zeros((1, 32), np.uint8), 5)


# --------------------------------------------------------------------- dequantize

@pytest.mark.parametrize("bits", [3, 4])
def test_dequantized_values_lie_on_group_grid(bits):
    N, K, g = 16, 512, 128
    W, A, B, _ = tiny_layer(N, K, 8, seed=21 + bits)
    codes, s, z = orc.quantize(W, A, B, bits, g)
    Wq = orc.dequant(orc.pack(codes, bits), s, z, K, bits, g)
    sd, zd = np.repeat(f64(s), g, axis=1), np.repeat(f64(z), g, axis=1)
    u = Wq / sd + zd
    assert np.all(np.abs(u - np.rint(u)) < 1e-9)
    assert np.all(np.rint(u) >= 0) and np.all(np.rint(u) <= 2 ** bits - 1)
    assert np.array_equal(np.rint(u).astype(np.uint8), codes)
    # and against numpy's own s*(q-z)
    assert np.allclose(Wq, sd * (codes.astype(np.float64) - zd), rtol=1e-15, atol=0)


# --------------------------------------------------------------------- y

def exact_y(x, codes, s, z, A, B, group):
    """y in exact rational arithmetic from the fp16 inputs (plain definition, triple loop)."""
    M, K = x.shape
    N = codes.shape[0]
    r = A.shape[1]
    F = lambda v: Fraction(float(v))
    y = [[Fraction(0)] * N for _ in range(M)]
    for m in range(M):
        t = [sum(F(x[m, k]) * F(A[k, j]) for k in range(K)) for j in range(r)]
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                acc += F(x[m, k]) * F(s[n, k // group]) * (int(codes[n, k]) - F(z[n, k // group]))
            acc += sum(t[j] * F(B[j, n]) for j in range(r))
            y[m][n] = acc
    return y


@pytest.mark.parametrize("bits,N,K,group,r", [(4, 8, 8, 8, 2), (3, 8, 32, 32, 3), (4, 4, 64, 32, 0)])
def test_linear_matches_exact_rational_arithmetic(bits, N, K, group, r):
    W, A, B, x = tiny_layer(N, K, r, seed=33 + bits, M=3)
    Aa, Bb = (A, B) if r else (None, None)
    codes, s, z = orc.quantize(W, Aa, Bb, bits, group)
    y = orc.linear(x, orc.pack(codes, bits), s, z, Aa, Bb, bits, group)
    ye = exact_y(x, codes, s, z, A, B, group)
    for m in range(x.shape[0]):
        for n in range(N):
            want = float(ye[m][n])
            assert abs(y[m, n] - want) <= 1e-13 * max(1.0, abs(want))


@pytest.mark.parametrize("bits", [3, 4])
def test_linear_two_routes_associativity_and_error_budget(bits):
    N, K, r, g, M = 48, 1024, 16, 128, 3
    W, A, B, x = tiny_layer(N, K, r, seed=44 + bits, M=M)
    codes, s, z = orc.quantize(W, A, B, bits, g)
    words = orc.pack(codes, bits)
    y = orc.linear(x, words, s, z, A, B, bits, g)
    WF = orc.reconstruct(words, s, z, A, B, K, bits, g)
    y2 = orc.dense_linear(x, WF)                                  # x.W_F^T with W_F materialised
    scale = np.linalg.norm(y)
    assert np.linalg.norm(y - y2) <= 1e-12 * scale
    y3 = f64(x) @ WF.T                                            # numpy GEMM
    assert np.linalg.norm(y - y3) <= 1e-12 * scale
    # (x.A).B against x.(A.B)
    Wq = orc.dequant(words, s, z, K, bits, g)
    y4 = f64(x) @ Wq.T + (f64(x) @ f64(A)) @ f64(B)
    assert np.linalg.norm(y - y4) <= 1e-12 * scale
    # Sec. 4.1 bound + Cauchy-Schwarz:  |y - x.W^T| <= ||x||_2 * (s_max/2) * sqrt(K)
    y_fp = f64(x) @ f64(W).T
    lim = np.linalg.norm(f64(x), axis=1)[:, None] * (f64(s).max(axis=1)[None, :] / 2) * np.sqrt(K)
    assert np.all(np.abs(y - y_fp) <= lim)


@pytest.mark.parametrize("bits", [3, 4])
def test_zero_up_projection_reduces_to_textbook_rtn_gemv(bits):
    """Alg. 1 initialises B = 0, so Sigma = 0 and the layer is the plain group-RTN quantized GEMV."""
    N, K, r, g = 24, 512, 8, 128
    W, A, _, x = tiny_layer(N, K, r, seed=55 + bits, M=2)
    B0 = np.zeros((r, N), np.float16)
    codes, s, z = orc.quantize(W, A, B0, bits, g)
    codes_plain, s_plain, z_plain = orc.quantize(W, None, None, bits, g)
    assert np.array_equal(codes, codes_plain) and np.array_equal(s, s_plain) and np.array_equal(z, z_plain)
    y = orc.linear(x, orc.pack(codes, bits), s, z, A, B0, bits, g)
    # textbook asymmetric min-max RTN in numpy (real-valued zero point), same fp16 storage of s and z
    qmax = 2 ** bits - 1
    Wg = f64(W).reshape(N, K // g, g)
    mn, mx = Wg.min(axis=2), Wg.max(axis=2)
    s_np = ((mx - mn) / qmax).astype(np.float16)
    z_np = (-mn / s_np.astype(np.float64)).astype(np.float16)
    assert np.array_equal(s_np, s) and np.array_equal(z_np, z)
    q_np = np.clip(np.rint(Wg / f64(s_np)[..., None] + f64(z_np)[..., None]), 0, qmax)
    W_rtn = (f64(s_np)[..., None] * (q_np - f64(z_np)[..., None])).reshape(N, K)
    assert np.array_equal(q_np.reshape(N, K).astype(np.uint8), codes)
    assert np.linalg.norm(y - f64(x) @ W_rtn.T) <= 1e-12 * np.linalg.norm(y)


@pytest.mark.parametrize("bits", [3, 4])
def test_unit_scale_zero_offset_is_exact_integer_arithmetic(bits):
    rng = np.random.Generator(np.random.Philox(66 + bits))
    N, K, g, M = 12, 256, 128, 4
    codes = rng.integers(0, 2 ** bits, (N, K), dtype=np.uint8)
    x = rng.integers(-2, 3, (M, K)).astype(np.float16)
    s = np.ones((N, K // g), np.float16)
    z = np.zeros((N, K // g), np.float16)
    y = orc.linear(x, orc.pack(codes, bits), s, z, None, None, bits, g)
    want = x.astype(np.int64) @ codes.astype(np.int64).T
    assert np.array_equal(y, want.astype(np.float64))


# --------------------------------------------------------------------- paper's printed figure

def test_sub_branch_mac_overhead_printed_by_the_paper():
    """Fig. 3 caption: M1/M0 = 2*b*r*d / (b*d*d) = 6.25 % at r = 128, d = 4096."""
    import os
    golden = os.path.join(os.path.dirname(__file__), "golden", "fig3_mac_overhead.txt")
    lines = [ln for ln in open(golden).read().splitlines() if ln and not ln.startswith("#")]
    fields = dict(tok.split("=") for ln in lines for tok in ln.split())
    d, r = int(fields["d"]), int(fields["r"])
    main = fbq_synth.algorithmic_flops(d, d, 0, 1)
    both = fbq_synth.algorithmic_flops(d, d, r, 1)
    assert abs((both - main) / main - float(fields["ratio"])) < 1e-12
