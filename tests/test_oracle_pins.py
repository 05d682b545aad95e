"""Pins of the CPU oracle against things other than itself.

Each test fixes one part of oracle/qbert_oracle.c to a value that the paper or plain
mathematics determines: closed-form lattices, exact rational arithmetic, brute force with
Python integers, numpy's own matmul/packbits, special cases of the grouping rule, and the
model sizes printed in Table 1.  None of them retypes the oracle's float32 formula.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

BITS = (2, 3, 4, 8)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def exact_levels(m, L):
    """The 2^k quantized points of the range [-m, m] as exact rationals (App.: q0 + Delta*j)."""
    m = Fraction(float(m))
    return [-m + (2 * m / L) * j for j in range(L + 1)]


# ---- P1: closed-form lattice --------------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("e", (-7, 0, 3))
def test_lattice_points_map_to_their_index(bits, e):
    L = 2 ** bits - 1
    h = np.float32(2.0 ** e)
    w = np.array([h * (2 * j - L) for j in range(L + 1)], np.float32)  # exact in fp32
    W = np.tile(w, (2, 3)).astype(np.float32)  # one group, 2 rows
    codes, hh, mm, rs = oracle.quantize_groupwise(W, bits, 1)
    assert mm[0] == h * L and hh[0] == h
    assert (codes == np.tile(np.arange(L + 1, dtype=np.uint8), (2, 3))).all()
    deq = oracle.dequantize_groupwise(codes, hh, bits)
    assert (deq == W.astype(np.float64)).all()
    # sum of (u - 2^(k-1)) over j = 0..L is -(L+1)/2 per period, 3 periods per row
    assert (rs == -3 * (L + 1) // 2).all()


# ---- P2: |w - Q(w)| <= Delta/2, and exact nearest-level property ---------------------------
@pytest.mark.parametrize("bits", BITS)
def test_error_bound_and_extremes(bits):
    L = 2 ** bits - 1
    W = (rng(1).standard_normal((24, 40)) * 0.04).astype(np.float32)
    W[3, 5] = 0.9  # an outlier
    G = 4
    codes, h, m, _ = oracle.quantize_groupwise(W, bits, G)
    deq = oracle.dequantize_groupwise(codes, h, bits)
    rows = 24 // G
    for g in range(G):
        blk = slice(g * rows, (g + 1) * rows)
        assert m[g] == np.abs(W[blk]).max()
        err = np.abs(W[blk].astype(np.float64) - deq[blk])
        assert err.max() <= float(h[g]) * (1 + 1e-6) + 4 * np.spacing(np.float64(m[g]).astype(np.float32))
        wb, cb = W[blk], codes[blk]
        assert set(np.unique(cb[np.abs(wb) == m[g]])) <= {0, L}
        assert (cb[wb == m[g]] == L).all() and (cb[wb == -m[g]] == 0).all()


@pytest.mark.parametrize("bits", BITS)
def test_code_is_nearest_exact_level(bits):
    """Exact rational arithmetic: the code is the index of the nearest of the 2^k levels."""
    L = 2 ** bits - 1
    W = (rng(2).standard_normal((6, 32)) * 0.3).astype(np.float32)
    codes, h, m, _ = oracle.quantize_groupwise(W, bits, 2)
    checked = 0
    for g in range(2):
        mg = Fraction(float(m[g]))
        for r in range(3 * g, 3 * g + 3):
            for j in range(32):
                t = (Fraction(float(W[r, j])) + mg) * L / (2 * mg)  # exact (w - q0)/Delta
                frac = t - (t.numerator // t.denominator)
                if abs(frac - Fraction(1, 2)) < Fraction(1, 10 ** 5):
                    continue  # too close to a decision boundary for float32 to be held to it
                assert codes[r, j] == int(round(t))
                checked += 1
    assert checked > 150


@pytest.mark.parametrize("bits", BITS)
def test_dequantized_value_is_the_exact_level(bits):
    """Q(w) = Delta*u + q0 evaluated exactly, against the oracle's h*(2u-L), to float32 accuracy."""
    L = 2 ** bits - 1
    W = (rng(3).standard_normal((4, 64))).astype(np.float32)
    codes, h, m, _ = oracle.quantize_groupwise(W, bits, 1)
    deq = oracle.dequantize_groupwise(codes, h, bits)
    lv = exact_levels(m[0], L)
    for r in range(4):
        for j in range(64):
            ex = lv[codes[r, j]]
            assert abs(Fraction(deq[r, j]) - ex) <= abs(ex) * Fraction(1, 2 ** 23)


# ---- P3: ties go to the even code; activation zero --------------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_ties_round_half_to_even(bits):
    L = 2 ** bits - 1
    h = np.float32(0.25)
    mids = np.array([h * (2 * j + 1 - L) for j in range(L)], np.float32)  # t = j + 1/2 exactly
    W = np.concatenate([[-h * L, h * L], mids]).astype(np.float32)[None, :]
    codes, hh, mm, _ = oracle.quantize_groupwise(W, bits, 1)
    assert hh[0] == h
    expect = np.array([j if j % 2 == 0 else j + 1 for j in range(L)], np.uint8)
    assert (codes[0, 2:] == expect).all()


def test_activation_special_values():
    clip = 6.0
    X = np.array([[0.0, -0.0, 6.0, -6.0, 100.0, -100.0, np.inf, -np.inf]], np.float32)
    xq, rs = oracle.quantize_act(X, clip)
    # x = 0 sits exactly between codes 127 and 128: half-to-even picks 128, stored 128-128 = 0
    assert xq[0].tolist() == [0, 0, 127, -128, 127, -128, 127, -128]
    assert rs[0] == sum(xq[0].tolist())


def test_activation_lattice_and_exact_nearest():
    clip = np.float32(255 / 64.0)  # h_x = 1/64 exactly
    u = np.arange(256)
    X = ((2 * u - 255) / 64.0).astype(np.float32)[None, :]
    xq, rs = oracle.quantize_act(X, float(clip))
    assert (xq[0].astype(np.int64) + 128 == u).all()
    Xh = oracle.dequantize_act(xq, float(clip))
    assert (Xh == X.astype(np.float64)).all()
    # random values: nearest of 256 exact levels
    X = (rng(4).standard_normal((3, 50)) * 2).astype(np.float32)
    xq, _ = oracle.quantize_act(X, 6.0)
    c = Fraction(6)
    for r in range(3):
        for j in range(50):
            x = min(max(Fraction(float(X[r, j])), -c), c)
            t = (x + c) * 255 / (2 * c)
            fr = t - (t.numerator // t.denominator)
            if abs(fr - Fraction(1, 2)) < Fraction(1, 10 ** 4):
                continue
            assert int(xq[r, j]) + 128 == int(round(t))


# ---- P4: idempotence ---------------------------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_quantize_dequantize_idempotent(bits):
    W = (rng(5).standard_normal((16, 48)) * 0.05).astype(np.float32)
    codes, h, m, _ = oracle.quantize_groupwise(W, bits, 4)
    Wq = oracle.dequantize_groupwise(codes, h, bits).astype(np.float32)
    codes2, h2, m2, _ = oracle.quantize_groupwise(Wq, bits, 4)
    assert (codes2 == codes).all()
    Wq2 = oracle.dequantize_groupwise(codes2, h2, bits).astype(np.float32)
    assert np.allclose(Wq2, Wq, rtol=3e-7, atol=0)


# ---- P5: code range and count --------------------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_code_range_and_all_levels_used(bits):
    L = 2 ** bits - 1
    W = rng(6).uniform(-1, 1, (8, 512)).astype(np.float32)
    codes, _, _, rs = oracle.quantize_groupwise(W, bits, 2)
    assert codes.max() <= L
    for g in range(2):
        assert len(np.unique(codes[4 * g:4 * g + 4])) == L + 1
    assert (rs == (codes.astype(np.int64) - 2 ** (bits - 1)).sum(1)).all()


def test_all_zero_group():
    W = np.zeros((4, 8), np.float32)
    W[2:] = 0.5
    codes, h, m, rs = oracle.quantize_groupwise(W, 4, 2)
    assert m[0] == 0 and h[0] == 0 and (codes[:2] == 0).all()
    assert (oracle.dequantize_groupwise(codes, h, 4)[:2] == 0).all()
    assert (codes[2:] == 15).all()


# ---- P6: special cases of the grouping rule (Fig. 3; Table 2's 1/12/128/768 groups) ---------------
@pytest.mark.parametrize("bits", (2, 4))
@pytest.mark.parametrize("G", (1, 12, 24, 128, 768))
def test_groups_equal_separately_quantized_row_blocks(bits, G):
    N, K = 768, 32
    W = (rng(7).standard_normal((N, K)) * 0.04).astype(np.float32)
    codes, h, m, rs = oracle.quantize_groupwise(W, bits, G)
    rows = N // G
    for g in (0, G // 2, G - 1):
        blk = slice(g * rows, (g + 1) * rows)
        c1, h1, m1, rs1 = oracle.quantize_groupwise(W[blk], bits, 1)
        assert (c1 == codes[blk]).all() and h1[0] == h[g] and m1[0] == m[g] and (rs1 == rs[blk]).all()
        assert m[g] == np.abs(W[blk]).max()
    if G == 768:  # one range per output neuron: per-channel quantization
        assert (m == np.abs(W).max(axis=1)).all()
    if G == 12:   # one range per head: blocks of d/N_h = 64 neurons
        assert rows == 64


# ---- P7 / P8: scale equivariance, monotonicity -------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_power_of_two_equivariance_and_monotone(bits):
    W = (rng(8).standard_normal((8, 64)) * 0.04).astype(np.float32)
    c1, h1, m1, _ = oracle.quantize_groupwise(W, bits, 2)
    c2, h2, m2, _ = oracle.quantize_groupwise(W * np.float32(16), bits, 2)
    assert (c1 == c2).all() and (h2 == h1 * 16).all() and (m2 == m1 * 16).all()
    for g in range(2):
        w = W[4 * g:4 * g + 4].ravel()
        c = c1[4 * g:4 * g + 4].ravel()
        order = np.argsort(w, kind="stable")
        assert (np.diff(c[order].astype(int)) >= 0).all()


# ---- P9: packing against numpy.packbits, and the paper's printed sizes ----------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_pack_matches_little_endian_bitstream(bits):
    codes = rng(9).integers(0, 2 ** bits, (5, 64), dtype=np.uint8)
    packed = oracle.pack(codes, bits)
    assert packed.shape == (5, 64 * bits // 8)
    bitsarr = ((codes[:, :, None] >> np.arange(bits)[None, None, :]) & 1).astype(np.uint8)
    ref = np.packbits(bitsarr.reshape(5, -1), axis=1, bitorder="little")
    assert (packed == ref).all()
    assert (oracle.unpack(packed, 64, bits) == codes).all()


def test_model_sizes_match_table_1():
    """Packed bytes = parameters * k / 8 reproduces the size columns of Table 1."""
    rows = {}
    with open(os.path.join(GOLDEN, "table1_sizes.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            wb, eb, total, enc = line.split()
            rows[wb] = (float(total), float(enc))
    MiB = 2.0 ** 20
    d, ffn, layers = 768, 3072, 12
    per_layer_matrix = 4 * d * d + 2 * d * ffn            # quantized matrix elements
    per_layer_all = per_layer_matrix + (4 * d + ffn + d) + 4 * d  # + biases + 2 LayerNorms
    assert per_layer_matrix == 7077888 and per_layer_all == 7087872
    enc_params = layers * per_layer_all
    assert abs(enc_params * 4 / MiB - rows["32"][1]) < 0.06
    K = 768
    for bits in BITS:
        # bytes of one packed row as the oracle lays it out
        assert oracle.packed_row_bytes(K, bits) * 8 == K * bits
        # printed to one decimal; the 2-bit row (20.4 against 20.28) is the loosest
        assert abs(enc_params * bits / 8 / MiB - rows[str(bits)][1]) < 0.15
    from paper_1909_05840_amd import workloads
    for key, table in (("2/3", workloads.PAPER_BITS_2_3), ("2/4", workloads.PAPER_BITS_2_4)):
        size = sum(per_layer_all * b / 8 for b in table["SST-2"]) / MiB
        assert abs(size - rows[key][1]) < 0.15
    emb_8bit = rows["8"][0] - rows["8"][1]
    for wb in ("4", "3", "2", "2/3", "2/4"):
        assert abs((rows[wb][0] - rows[wb][1]) - emb_8bit) < 0.11  # every row carries the same 8-bit embedding


# ---- P10: brute-force integer product ------------------------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("G", (1, 2, 6))
def test_integer_product_brute_force(bits, G):
    T, N, K = 5, 6, 9
    L = 2 ** bits - 1
    r = rng(10 + bits)
    xq = r.integers(-128, 128, (T, K)).astype(np.int8)
    xq[0, :] = -128
    xq[1, :] = 127
    codes = r.integers(0, L + 1, (N, K)).astype(np.uint8)
    codes[0, :] = L
    codes[1, :] = 0
    h = (r.uniform(0.001, 0.01, G)).astype(np.float32)
    clip = 6.0
    Y, A4, acc = oracle.qlinear_fwd(xq, clip, codes, h, bits)
    hx = Fraction(float(np.float32(clip) / np.float32(255)))
    for t in range(T):
        for n in range(N):
            a4 = sum((2 * int(xq[t, j]) + 1) * (2 * int(codes[n, j]) - L) for j in range(K))
            a = sum(int(xq[t, j]) * (int(codes[n, j]) - 2 ** (bits - 1)) for j in range(K))
            assert A4[t, n] == a4 and acc[t, n] == a
            y = hx * Fraction(float(h[n // (N // G)])) * a4
            assert abs(Fraction(float(Y[t, n])) - y) <= abs(y) * Fraction(1, 2 ** 23)
    ts = np.array([0, 4, 2], np.int64)
    ns = np.array([5, 0, 3], np.int64)
    Ys, A4s = oracle.qlinear_fwd_sampled(xq, clip, codes, h, bits, ts, ns)
    assert (A4s == A4[ts, ns]).all() and (Ys == Y[ts, ns]).all()


# ---- P11: the layer equals a textbook GEMM on the de-quantized operands ----------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_forward_and_backward_equal_fp64_gemm(bits):
    T, N, K, G = 33, 24, 64, 4
    W = (rng(20).standard_normal((N, K)) * 0.04).astype(np.float32)
    X = rng(21).standard_normal((T, K)).astype(np.float32)
    bias = rng(22).standard_normal(N).astype(np.float32)
    codes, h, m, rs_w = oracle.quantize_groupwise(W, bits, G)
    xq, rs_x = oracle.quantize_act(X, 6.0)
    What = oracle.dequantize_groupwise(codes, h, bits)
    Xhat = oracle.dequantize_act(xq, 6.0)
    Y, A4, acc = oracle.qlinear_fwd(xq, 6.0, codes, h, bits)
    ref = Xhat @ What.T
    assert np.abs(Y - ref).max() <= 1e-6 * np.abs(ref).max()
    assert np.allclose(Y, ref, rtol=1e-6, atol=1e-9)
    assert (A4 == 4 * acc.astype(np.int64) + 2 * rs_x[:, None] + 2 * rs_w[None, :] + K).all()
    Yb, _, _ = oracle.qlinear_fwd(xq, 6.0, codes, h, bits, bias=bias)
    assert np.allclose(Yb, ref + bias[None, :], rtol=1e-6, atol=1e-7)
    # quantization error of the whole layer is small at 8 bits (sanity of the operand roles)
    if bits == 8:
        full = X.astype(np.float64) @ W.astype(np.float64).T
        assert np.linalg.norm(ref - full) / np.linalg.norm(full) < 0.05
    # backward: gradients of a plain GEMM
    dYf = (rng(23).standard_normal((T, N)) * 1e-2).astype(np.float32)
    dY_bits = (dYf.view(np.uint32) >> 16).astype(np.uint16)  # truncation is a valid bf16 value
    dY = (dY_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    dX, dW = oracle.qlinear_bwd_ste(dY_bits, xq, 6.0, codes, h, bits)
    assert np.allclose(dX, dY @ What, rtol=1e-12, atol=1e-15)
    assert np.allclose(dW, dY.T @ Xhat, rtol=1e-12, atol=1e-15)
    ts = np.array([0, 32, 7]); js = np.array([63, 0, 11]); ns = np.array([23, 0, 5])
    assert np.allclose(oracle.bwd_dx_sampled(dY_bits, codes, h, bits, ts, js), dX[ts, js], rtol=1e-12)
    assert np.allclose(oracle.bwd_dw_sampled(dY_bits, xq, 6.0, ns, js), dW[ns, js], rtol=1e-12)
    # finite-difference check of the STE reading: d<Y,dY>/dXhat = dX, d<Y,dY>/dWhat = dW
    eps = 1e-3
    E = np.zeros_like(Xhat); E[3, 5] = eps
    num = (((Xhat + E) @ What.T - ref) * dY).sum() / eps
    assert abs(num - dX[3, 5]) <= 1e-9 + 1e-6 * abs(dX[3, 5])


# ---- 8-bit output: forward followed at once by the activation quantizer ------------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_q8_output_exact_when_scales_are_powers_of_two(bits):
    """h_x = 2^-6 and h_g = 2^-e make y = h_x*h_g*A4 exact in binary32 and binary64 alike, so the fused
    result must equal the activation quantizer applied to the separately computed Y, bit for bit."""
    T, N, K, G = 9, 12, 64, 3
    L = 2 ** bits - 1
    r = rng(40 + bits)
    xq = r.integers(-128, 128, (T, K)).astype(np.int8)
    codes = r.integers(0, L + 1, (N, K)).astype(np.uint8)
    h = np.array([2.0 ** -9, 2.0 ** -8, 2.0 ** -10], np.float32)
    clip = np.float32(255 * 2.0 ** -6)
    assert np.float32(clip) / np.float32(255) == np.float32(2.0 ** -6)
    bias = (r.integers(-64, 64, N) * 2.0 ** -10).astype(np.float32)
    for b in (None, bias):
        Y, A4, _ = oracle.qlinear_fwd(xq, clip, codes, h, bits, bias=b)
        assert np.abs(A4).max() < 2 ** 24
        for clip_out in (0.5, 2.0, 6.0):
            yq, rs_y = oracle.qlinear_fwd_q8(xq, clip, codes, h, bits, clip_out, bias=b)
            ref_q, ref_rs = oracle.quantize_act(Y, clip_out)
            assert (yq == ref_q).all() and (rs_y == ref_rs).all()
            assert (rs_y == yq.astype(np.int64).sum(axis=1)).all()
    # a zero output is the tie 127.5 and rounds to the even code 128, stored as 0
    yq0, rs0 = oracle.qlinear_fwd_q8(np.zeros((2, K), np.int8), clip, np.full((N, K), 2 ** (bits - 1), np.uint8), h, bits, 6.0)
    y0, a40, _ = oracle.qlinear_fwd(np.zeros((2, K), np.int8), clip, np.full((N, K), 2 ** (bits - 1), np.uint8), h, bits)
    assert (yq0 == oracle.quantize_act(y0, 6.0)[0]).all()


@pytest.mark.parametrize("bits", (3, 8))
def test_q8_output_is_nearest_level_of_the_exact_product(bits):
    """Generic scales: the code's level is within half a step (plus rounding slack) of the exact rational
    h_x*h_g*A4 + bias clamped to the range, and it differs from the two-step route by at most one code."""
    T, N, K, G = 17, 24, 128, 4
    W = (rng(50).standard_normal((N, K)) * 0.04).astype(np.float32)
    X = rng(51).standard_normal((T, K)).astype(np.float32)
    bias = (rng(52).standard_normal(N) * 0.1).astype(np.float32)
    codes, h, m, rs_w = oracle.quantize_groupwise(W, bits, G)
    xq, rs_x = oracle.quantize_act(X, 6.0)
    clip_out = 0.5
    yq, rs_y = oracle.qlinear_fwd_q8(xq, 6.0, codes, h, bits, clip_out, bias=bias)
    Y, A4, _ = oracle.qlinear_fwd(xq, 6.0, codes, h, bits, bias=bias)
    two_step, _ = oracle.quantize_act(Y, clip_out)
    d = np.abs(yq.astype(np.int32) - two_step.astype(np.int32))
    assert d.max() <= 1 and (d != 0).mean() < 5e-3
    assert (rs_y == yq.astype(np.int64).sum(axis=1)).all()
    hx = Fraction(float(np.float32(6.0) / np.float32(255)))
    ho = Fraction(float(np.float32(clip_out) / np.float32(255)))
    c = Fraction(clip_out)
    for t in range(T):
        for n in range(N):
            y = hx * Fraction(float(h[n // (N // G)])) * int(A4[t, n]) + Fraction(float(bias[n]))
            y = max(-c, min(c, y))
            level = ho * (2 * (int(yq[t, n]) + 128) - 255)
            assert abs(level - y) <= ho * (1 + Fraction(1, 10 ** 4))
    assert yq.min() == -128 and yq.max() == 127  # the range is hit on both sides with this clip


def test_q8_output_gelu_matches_an_independent_erf():
    from scipy.special import erf
    T, N, K, G, bits = 16, 32, 64, 4, 4
    W = (rng(60).standard_normal((N, K)) * 0.04).astype(np.float32)
    X = rng(61).standard_normal((T, K)).astype(np.float32)
    codes, h, m, rs_w = oracle.quantize_groupwise(W, bits, G)
    xq, rs_x = oracle.quantize_act(X, 6.0)
    _, A4, _ = oracle.qlinear_fwd(xq, 6.0, codes, h, bits)
    hx = np.float32(6.0) / np.float32(255)
    y = (hx * np.repeat(h, N // G)[None, :]).astype(np.float32) * A4.astype(np.float32)  # binary32 steps
    assert y.dtype == np.float32
    g = (0.5 * y.astype(np.float64) * (1.0 + erf(y.astype(np.float64) / np.sqrt(2.0)))).astype(np.float32)
    ref_q, ref_rs = oracle.quantize_act(g, 1.0)
    yq, rs_y = oracle.qlinear_fwd_q8(xq, 6.0, codes, h, bits, 1.0, act=1)
    d = np.abs(yq.astype(np.int32) - ref_q.astype(np.int32))
    assert d.max() <= 1 and (d != 0).mean() < 1e-3
    assert (rs_y == yq.astype(np.int64).sum(axis=1)).all()
    # GELU's shape: never below -0.17, identity-like for large positive inputs
    lev = (np.float64(1.0) / 255) * (2 * (yq.astype(np.int64) + 128) - 255)
    assert lev.min() >= -0.17 - 1.0 / 255
    big = y > 0.9
    assert big.any() and np.abs(lev[big] - np.minimum(g[big], 1.0)).max() <= 1.0 / 255 * 1.001


# ---- clipped weight ranges ------------------------------------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_clipped_group_range(bits):
    """A given range equal to the max-abs reproduces the plain quantizer; a smaller one clamps: weights outside get
    the end codes, weights inside get the nearest level of the exact quotient; the end codes de-quantize to -+m."""
    N, K, G = 12, 64, 4
    L = 2 ** bits - 1
    W = (rng(80 + bits).standard_normal((N, K)) * 0.04).astype(np.float32)
    codes, h, m, rs_w = oracle.quantize_groupwise(W, bits, G)
    c2, h2, rs2 = oracle.quantize_groupwise_clip(W, bits, m)
    assert (c2 == codes).all() and (h2 == h).all() and (rs2 == rs_w).all()
    mc = (0.5 * m).astype(np.float32)
    c3, h3, rs3 = oracle.quantize_groupwise_clip(W, bits, mc)
    assert (rs3 == (c3.astype(np.int64) - 2 ** (bits - 1)).sum(axis=1)).all()
    rows = N // G
    clipped = 0
    for n in range(N):
        mg, hg = Fraction(float(mc[n // rows])), Fraction(float(h3[n // rows]))
        assert hg == Fraction(float(np.float32(mc[n // rows]) / np.float32(L)))
        for j in range(K):
            w = Fraction(float(W[n, j]))
            u = int(c3[n, j])
            if w >= mg:
                assert u == L
                clipped += 1
            elif w <= -mg:
                assert u == 0
                clipped += 1
            else:
                assert abs(hg * (2 * u - L) - w) <= hg * (1 + Fraction(1, 10 ** 5))
    assert clipped > 0
    # m = 0: everything is code 0, h = 0
    c4, h4, _ = oracle.quantize_groupwise_clip(W, bits, np.zeros(G, np.float32))
    assert (c4 == 0).all() and (h4 == 0).all()


# ---- dynamic (per-token max-abs) activation range ---------------------------------------------------------------
def test_dynamic_activation_range_equals_static_quantizer_row_by_row():
    """Each row is the static quantizer with clip = that row's max-abs; the row's extreme hits code 0 or 255; the
    forward with per-token scales equals the fp64 GEMM of the de-quantized operands."""
    T, K, N, G, bits = 13, 64, 12, 3, 4
    X = rng(70).standard_normal((T, K)).astype(np.float32)
    X[3] *= 100.0
    X[5] = 0.0
    X[7] = 2.0 ** -20 * X[7]
    xq, rs, hx = oracle.quantize_act_dyn(X)
    for t in range(T):
        c = float(np.abs(X[t]).max())
        if c == 0.0:
            assert hx[t] == 0 and (xq[t] == -128).all() and rs[t] == -128 * K   # code 0 everywhere, like a zero group
            continue
        q1, r1 = oracle.quantize_act(X[t:t + 1], c)
        assert (xq[t] == q1[0]).all() and rs[t] == r1[0]
        assert hx[t] == np.float32(c) / np.float32(255)
        assert xq[t].max() == 127 or xq[t].min() == -128
        # nearest level of the exact quotient
        lev = float(hx[t]) * (2 * (xq[t].astype(np.int64) + 128) - 255)
        assert np.abs(lev - X[t].astype(np.float64)).max() <= float(hx[t]) * (1 + 1e-5)
    W = (rng(71).standard_normal((N, K)) * 0.04).astype(np.float32)
    codes, h, m, rs_w = oracle.quantize_groupwise(W, bits, G)
    bias = rng(72).standard_normal(N).astype(np.float32)
    Y, A4 = oracle.qlinear_fwd_dyn(xq, hx, codes, h, bits)
    What = oracle.dequantize_groupwise(codes, h, bits)
    Xhat = hx.astype(np.float64)[:, None] * (2 * xq.astype(np.float64) + 1)
    ref = Xhat @ What.T
    assert np.allclose(Y, ref, rtol=1e-6, atol=1e-30)
    assert (Y[5] == 0).all() and (A4[5] != 0).any()      # zero row: zero scale times a non-zero integer
    Yb, _ = oracle.qlinear_fwd_dyn(xq, hx, codes, h, bits, bias=bias)
    assert np.allclose(Yb, ref + bias[None, :], rtol=1e-6, atol=1e-7)
    # a constant per-token scale reproduces the static forward bit for bit
    xs, rss = oracle.quantize_act(X, 6.0)
    Ys, A4s, _ = oracle.qlinear_fwd(xs, 6.0, codes, h, bits)
    hconst = np.full(T, np.float32(6.0) / np.float32(255), np.float32)
    Yd, A4d = oracle.qlinear_fwd_dyn(xs, hconst, codes, h, bits)
    assert (Yd == Ys).all() and (A4d == A4s).all()


# ---- P12: backward is linear in dY ---------------------------------------------------------------------------------
def test_backward_linearity():
    T, N, K = 8, 6, 16
    r = rng(30)
    xq = r.integers(-128, 128, (T, K)).astype(np.int8)
    codes = r.integers(0, 8, (N, K)).astype(np.uint8)
    h = r.uniform(0.01, 0.02, 2).astype(np.float32)

    def bf(x):  # exact bf16 values: small integers / 64
        return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)
    d1 = r.integers(-8, 9, (T, N)) / 64.0
    d2 = r.integers(-8, 9, (T, N)) / 64.0
    a = 2.0
    X1, W1 = oracle.qlinear_bwd_ste(bf(d1), xq, 6.0, codes, h, 3)
    X2, W2 = oracle.qlinear_bwd_ste(bf(d2), xq, 6.0, codes, h, 3)
    X3, W3 = oracle.qlinear_bwd_ste(bf(a * d1 + d2), xq, 6.0, codes, h, 3)
    assert np.allclose(X3, a * X1 + X2, rtol=1e-12, atol=1e-15)
    assert np.allclose(W3, a * W1 + W2, rtol=1e-12, atol=1e-15)


# ---- P13: embedding = weight quantizer on the transposed table; gather = row select -----------------------------------
@pytest.mark.parametrize("bits", (4, 8))
def test_embedding_is_weight_grouping_on_transpose(bits):
    V, d, G = 50, 32, 8
    E = (rng(40).standard_normal((V, d)) * 0.02).astype(np.float32)
    codes, h, m = oracle.embedding_quantize(E, G, bits)
    cT, hT, mT, _ = oracle.quantize_groupwise(np.ascontiguousarray(E.T), bits, G)
    assert (codes == cT.T).all() and (h == hT).all() and (m == mT).all()
    cols = d // G
    for g in range(G):
        assert m[g] == np.abs(E[:, g * cols:(g + 1) * cols]).max()
    ids = np.array([3, 3, 49, 0, 17], np.int64)
    out = oracle.embedding_gather(codes, h, ids, bits)
    full = oracle.dequantize_groupwise(cT, hT, bits).T
    assert (out == full[ids]).all()
    assert np.abs(out - E[ids]).max() <= h.max() * (1 + 1e-6)
    assert codes.max() == 2 ** bits - 1 and codes.min() == 0


def test_mixed_precision_embedding_size_matches_the_paper():
    """App. "Mixed Precision Quantization for Embedding": 4-bit word and 8-bit position embeddings bring the
    embedding table to 11.6 MB (about 8x smaller than the 91 MB of fp32); sizes from the packed row lengths."""
    d = 768
    word, pos, typ = 30522 * d, 512 * d, 2 * d
    mib = 2.0 ** 20
    fp32 = (word + pos + typ) * 4 / mib
    assert abs(fp32 - 91.0) < 0.5                                   # Sec. 3: 91 MB for the embedding
    mixed = (30522 * oracle.packed_row_bytes(d, 4) + 512 * oracle.packed_row_bytes(d, 8) + 2 * oracle.packed_row_bytes(d, 8)) / mib
    assert abs(mixed - 11.6) < 0.06
    assert 7.5 < fp32 / mixed < 8.1
    assert abs((word + pos + typ) / mib - fp32 / 4) < 1e-9           # all 8 bits: the 4x of the abstract


def test_argument_errors():
    W = np.zeros((6, 8), np.float32)
    with pytest.raises(oracle.OracleError):
        oracle.quantize_groupwise(W, 5, 2)
    with pytest.raises(oracle.OracleError):
        oracle.quantize_groupwise(W, 4, 4)  # 6 rows do not split into 4 groups
    W[0, 0] = np.nan
    with pytest.raises(oracle.OracleError):
        oracle.quantize_groupwise(W, 4, 2)
    with pytest.raises(oracle.OracleError):
        oracle.quantize_act(np.zeros((2, 2), np.float32), -1.0)


def test_dynamic_tensor_range_worked_example_and_special_cases():
    """One range for the whole tensor, c = max|X| (App. A: any range [q0, q_255]).  A case worked by hand with
    c = 31.875, h = 1/8, Delta = 1/4 (every quotient exact); the static quantizer at clip = c; the nearest-level
    bound; a zero tensor; the forward against the fp64 product of the de-quantized operands."""
    X = np.array([[-31.875, 0.125, 10.125, -0.125], [31.875, -0.125, 0.125, -31.625]], np.float32)
    xq, rs, hx = oracle.quantize_act_dyn_tensor(X)
    assert hx == np.float32(0.125)
    assert xq.tolist() == [[-128, 0, 40, -1], [127, -1, 0, -127]]
    assert rs.tolist() == [-89, -1]

    T, K, N, G, bits = 9, 64, 8, 2, 3
    X = rng(90).standard_normal((T, K)).astype(np.float32)
    X[2] *= 50.0          # the tensor's maximum sits in row 2: the other rows use few of the 256 levels
    c = float(np.abs(X).max())
    xq, rs, hx = oracle.quantize_act_dyn_tensor(X)
    q1, r1 = oracle.quantize_act(X, c)
    assert (xq == q1).all() and (rs == r1).all() and hx == np.float32(c) / np.float32(255)
    assert xq.max() == 127 or xq.min() == -128
    lev = float(hx) * (2 * (xq.astype(np.int64) + 128) - 255)
    assert np.abs(lev - X.astype(np.float64)).max() <= float(hx) * (1 + 1e-5)
    others = np.delete(np.arange(T), 2)
    assert np.unique(xq[others]).size < 40                     # coarse for the small rows ...
    xq_t, _, hx_t = oracle.quantize_act_dyn(X)
    assert np.unique(xq_t[others]).size > 150                  # ... unlike a range per token
    assert (xq_t[2] == xq[2]).all() and hx_t[2] == hx

    W = (rng(91).standard_normal((N, K)) * 0.04).astype(np.float32)
    codes, h, m, rs_w = oracle.quantize_groupwise(W, bits, G)
    Y, A4 = oracle.qlinear_fwd_dyn(xq, np.full(T, hx, np.float32), codes, h, bits)
    Y1, A41, _ = oracle.qlinear_fwd(xq, c, codes, h, bits)
    assert (A4 == A41).all() and (Y == Y1).all()
    ref = (float(hx) * (2 * xq.astype(np.float64) + 1)) @ oracle.dequantize_groupwise(codes, h, bits).T
    assert np.allclose(Y, ref, rtol=1e-6, atol=1e-30)

    Z = np.zeros((3, 32), np.float32)
    xq, rs, hx = oracle.quantize_act_dyn_tensor(Z)
    assert hx == 0 and (xq == -128).all() and (rs == -128 * 32).all()
    Z[1, 5] = np.inf
    with pytest.raises(Exception):
        oracle.quantize_act_dyn_tensor(Z)


def test_masked_ste_is_the_gradient_of_the_clamped_layer():
    """With only the rounding passed straight through, the layer is <dY, Clamp(X) What^T> in X and
    <dY, Xhat Clamp_g(W)^T> in W: the masked backward must equal central differences of those (fp64, away from the
    kinks), be exactly zero outside the ranges and untouched inside, pass at the range's ends, and equal the plain
    backward when nothing lies outside."""
    T, N, K, G, bits = 7, 8, 64, 2, 4
    clip = 1.5
    X = rng(95).standard_normal((T, K)).astype(np.float32)
    X[0, 0], X[0, 1], X[0, 2] = clip, -clip, np.nextafter(np.float32(clip), np.float32(2))
    W = (rng(96).standard_normal((N, K)) * 0.05).astype(np.float32)
    m = np.array([0.06, np.abs(W[N // 2:]).max()], np.float32)      # group 0 clipped, group 1 at its max-abs
    W[1, 3] = -m[0]
    codes, h, rs_w = oracle.quantize_groupwise_clip(W, bits, m)
    xq, rs_x = oracle.quantize_act(X, clip)
    dYf = (rng(97).standard_normal((T, N)) * 1e-2).astype(np.float32)
    dY_bits = (dYf.view(np.uint32) >> 16).astype(np.uint16)
    dY = (dY_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    dX, dW = oracle.qlinear_bwd_ste(dY_bits, xq, clip, codes, h, bits)
    dXm, dWm = oracle.qlinear_bwd_ste_masked(dY_bits, xq, clip, codes, h, bits, X=X, W=W, m=m)
    outX = np.abs(X) > np.float32(clip)
    mrow = np.repeat(m, N // G)[:, None]
    outW = np.abs(W) > mrow
    assert outX.sum() > 20 and outW[:N // 2].sum() > 20 and not outW[N // 2:].any()
    assert not outX[0, 0] and not outX[0, 1] and outX[0, 2] and not outW[1, 3]
    assert (dXm[outX] == 0).all() and (dXm[~outX] == dX[~outX]).all() and (dX[outX] != 0).all()
    assert (dWm[outW] == 0).all() and (dWm[~outW] == dW[~outW]).all() and (dW[outW] != 0).all()
    # only one side masked
    a, b = oracle.qlinear_bwd_ste_masked(dY_bits, xq, clip, codes, h, bits, X=X)
    assert (a == dXm).all() and (b == dW).all()
    a, b = oracle.qlinear_bwd_ste_masked(dY_bits, xq, clip, codes, h, bits, W=W, m=m)
    assert (a == dX).all() and (b == dWm).all()
    # central differences of the clamped layer
    What = oracle.dequantize_groupwise(codes, h, bits)
    Xhat = oracle.dequantize_act(xq, clip)
    X64, W64 = X.astype(np.float64), W.astype(np.float64)
    fX = lambda Xv: ((np.clip(Xv, -clip, clip) @ What.T) * dY).sum()
    fW = lambda Wv: ((Xhat @ np.clip(Wv, -mrow.astype(np.float64), mrow.astype(np.float64)).T) * dY).sum()
    eps = 1e-4
    r = rng(98)
    checked_out = 0
    for _ in range(60):
        t, j = r.integers(0, T), r.integers(0, K)
        if abs(abs(X64[t, j]) - clip) > 1e-2:
            E = np.zeros_like(X64); E[t, j] = eps
            num = (fX(X64 + E) - fX(X64 - E)) / (2 * eps)
            assert abs(num - dXm[t, j]) <= 1e-10 + 1e-6 * abs(dX[t, j])
            checked_out += int(outX[t, j])
        n, j = r.integers(0, N), r.integers(0, K)
        if abs(abs(W64[n, j]) - float(mrow[n, 0])) > 1e-3:
            E = np.zeros_like(W64); E[n, j] = eps
            num = (fW(W64 + E) - fW(W64 - E)) / (2 * eps)
            assert abs(num - dWm[n, j]) <= 1e-10 + 1e-6 * abs(dW[n, j])
            checked_out += int(outW[n, j])
    assert checked_out >= 5
    # nothing outside: the plain backward
    Xs = (0.1 * X).astype(np.float32)
    xqs, _ = oracle.quantize_act(Xs, clip)
    c2, h2, m2, _ = oracle.quantize_groupwise(W, bits, G)
    p = oracle.qlinear_bwd_ste(dY_bits, xqs, clip, c2, h2, bits)
    q = oracle.qlinear_bwd_ste_masked(dY_bits, xqs, clip, c2, h2, bits, X=Xs, W=W, m=m2)
    assert (p[0] == q[0]).all() and (p[1] == q[1]).all()


# ---- asymmetric group ranges [min, max] (App. A, general q0) ----------------------------------------------------------
@pytest.mark.parametrize("bits", BITS)
def test_asymmetric_range_lattice_nearest_level_and_special_cases(bits):
    """Closed-form lattice (weights on q0 + Delta*u come back as u, de-quantize exactly), nearest level by exact
    rational arithmetic, both ends of the range are codes 0 and L, all levels used; a symmetric group gives the
    symmetric quantizer's codes; a constant group has Delta = 0, codes 0 and Q = q0; an all-positive group spends
    no level on negative values."""
    from fractions import Fraction
    L = 2 ** bits - 1
    # lattice: q0 = -0.75, Delta = 2^-5: exact in binary32
    K = 64
    u = (np.arange(2 * K) * 7 % (L + 1)).reshape(2, K)
    u[0, 0], u[1, 1] = 0, L
    W = (-0.75 + u * 2.0 ** -5).astype(np.float32)
    codes, delta, q0, rs = oracle.quantize_groupwise_asym(W, bits, 1)
    assert delta[0] == np.float32(2.0 ** -5) and q0[0] == np.float32(-0.75)
    assert (codes == u).all()
    assert (rs == (u - 2 ** (bits - 1)).sum(axis=1)).all()
    assert (oracle.dequantize_groupwise_asym(codes, delta, q0) == W.astype(np.float64)).all()
    # random data, two groups with different offsets
    r = rng(110 + bits)
    W = np.concatenate([r.uniform(0.1, 0.9, (3, K)), r.normal(-2.0, 0.3, (3, K))]).astype(np.float32)
    codes, delta, q0, rs = oracle.quantize_groupwise_asym(W, bits, 2)
    for g in range(2):
        Wg, cg = W[3 * g:3 * g + 3], codes[3 * g:3 * g + 3]
        assert q0[g] == Wg.min() and delta[g] == np.float32(np.float32(Wg.max() - Wg.min()) / np.float32(L))
        assert cg[Wg == Wg.min()].max() == 0 and cg[Wg == Wg.max()].min() == L
        if bits <= 4 and g == 0:                                   # uniform data: every level occurs
            assert np.unique(cg).size == L + 1
        d, z = Fraction(float(delta[g])), Fraction(float(q0[g]))
        for w, c in zip(Wg.ravel()[:60], cg.ravel()[:60]):
            err = abs(Fraction(float(w)) - (d * int(c) + z))
            assert err <= d / 2 * (1 + Fraction(1, 10 ** 5))       # nearest of the levels (up to binary32 rounding)
    assert (q0[0] > 0) and codes[:3].min() == 0                     # all-positive group: level 0 is its minimum
    # symmetric group: same codes as the symmetric quantizer
    Ws = r.standard_normal((4, K)).astype(np.float32)
    Ws[0, 0] = -np.abs(Ws).max() * 1.5
    Ws[1, 1] = -Ws[0, 0]
    ca, da, qa, rsa = oracle.quantize_groupwise_asym(Ws, bits, 1)
    cs, hs, ms, rss = oracle.quantize_groupwise(Ws, bits, 1)
    assert qa[0] == -ms[0] and (ca == cs).all() and (rsa == rss).all()
    # constant group
    Wc = np.full((2, K), 0.3, np.float32)
    cc, dc, qc, rc = oracle.quantize_groupwise_asym(Wc, bits, 1)
    assert dc[0] == 0 and qc[0] == np.float32(0.3) and (cc == 0).all()
    assert (oracle.dequantize_groupwise_asym(cc, dc, qc) == float(np.float32(0.3))).all()
    assert (rc == -K * 2 ** (bits - 1)).all()


@pytest.mark.parametrize("bits", BITS)
def test_asymmetric_forward_and_backward_equal_fp64_gemm(bits):
    """Y and dX against numpy fp64 products of the de-quantized operands; the integer sum S by Python integers; on a
    symmetric group the result agrees with the symmetric forward; the error of the layer is smaller than the
    symmetric quantizer's on one-sided weights (what the wider use of the levels buys)."""
    T, N, K, G = 11, 12, 64, 3
    r = rng(120 + bits)
    W = (r.uniform(0.0, 0.08, (N, K))).astype(np.float32)      # one-sided, like weights after a ReLU-style shift
    X = r.standard_normal((T, K)).astype(np.float32)
    bias = r.standard_normal(N).astype(np.float32)
    codes, delta, q0, rs_w = oracle.quantize_groupwise_asym(W, bits, G)
    xq, rs_x = oracle.quantize_act(X, 6.0)
    What = oracle.dequantize_groupwise_asym(codes, delta, q0)
    Xhat = oracle.dequantize_act(xq, 6.0)
    Y, S = oracle.qlinear_fwd_asym(xq, 6.0, codes, delta, q0, want_s=True)
    ref = Xhat @ What.T
    scale = (np.abs(Xhat) @ np.abs(What).T)
    assert (np.abs(Y - ref) <= 1e-6 * scale).all()
    xi = 2 * xq.astype(object) + 1
    assert S[3, 5] == sum(int(a) * int(c) for a, c in zip(xi[3], codes[5]))
    assert S[10, 11] == sum(int(a) * int(c) for a, c in zip(xi[10], codes[11]))
    Yb = oracle.qlinear_fwd_asym(xq, 6.0, codes, delta, q0, bias=bias)
    assert (np.abs(Yb - (ref + bias[None, :])) <= 1e-6 * (scale + np.abs(bias)[None, :])).all()
    dYf = (r.standard_normal((T, N)) * 1e-2).astype(np.float32)
    dY_bits = (dYf.view(np.uint32) >> 16).astype(np.uint16)
    dY = (dY_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    dX = oracle.qlinear_bwd_dx_asym(dY_bits, codes, delta, q0)
    assert np.allclose(dX, dY @ What, rtol=1e-12, atol=1e-15)
    # less layer error than the symmetric range on one-sided weights
    cs, hs, ms, _ = oracle.quantize_groupwise(W, bits, G)
    full = Xhat @ W.astype(np.float64).T
    e_asym = np.linalg.norm(ref - full)
    e_sym = np.linalg.norm(Xhat @ oracle.dequantize_groupwise(cs, hs, bits).T - full)
    assert e_asym < 0.7 * e_sym
    # symmetric groups: the two forwards agree
    Wsym = r.standard_normal((N, K)).astype(np.float32) * 0.05
    for g in range(G):
        blk = Wsym[g * (N // G):(g + 1) * (N // G)]
        mval = np.abs(blk).max()
        blk[0, 0], blk[0, 1] = mval, -mval
    ca, da, qa, _ = oracle.quantize_groupwise_asym(Wsym, bits, G)
    cs, hs, ms, _ = oracle.quantize_groupwise(Wsym, bits, G)
    assert (ca == cs).all()
    Ya = oracle.qlinear_fwd_asym(xq, 6.0, ca, da, qa)
    Ys, _, _ = oracle.qlinear_fwd(xq, 6.0, cs, hs, bits)
    sc = np.abs(Xhat) @ np.abs(oracle.dequantize_groupwise(cs, hs, bits)).T
    assert (np.abs(Ya - Ys) <= 2e-6 * sc).all()


# ---- Hessian sensitivity: Eq. 2 and Alg. 1 -------------------------------------------------------------------------
def test_sensitivity_omega_and_power_iteration():
    """Eq. 2 on cases worked by hand; the ranking; Alg. 1 against a symmetric matrix built from a known spectrum (the
    estimate converges to the eigenvalue of largest magnitude, sign included, at the rate (l2/l1)^2 per step, and v to
    its eigenvector) and against numpy's eigensolver."""
    om = oracle.sensitivity_omega([[1.0, 3.0], [-1.0, -3.0], [2.0, 2.0], [-4.0, 4.0]])
    assert np.allclose(om, [3.0, 3.0, 2.0, 4.0], rtol=0, atol=1e-15)       # mean 2, std 1 | mean -2 | constant | mean 0, std 4
    assert oracle.rank_by_sensitivity(om).tolist() == [3, 0, 1, 2]          # descending, ties in layer order
    r = rng(130)
    n = 40
    Q, _ = np.linalg.qr(r.standard_normal((n, n)))
    spec = np.concatenate([[-5.0, 3.0], r.uniform(-2.0, 2.0, n - 2)])      # the top eigenvalue is negative
    H = (Q * spec) @ Q.T
    H = 0.5 * (H + H.T)
    lam, v = oracle.power_iteration(lambda x: H @ x, r.standard_normal(n), 60)
    assert abs(lam[-1] + 5.0) < 1e-9
    assert min(np.abs(v - Q[:, 0]).max(), np.abs(v + Q[:, 0]).max()) < 1e-6
    w = np.linalg.eigvalsh(H)
    assert abs(lam[-1] - w[np.argmax(np.abs(w))]) < 1e-9
    err = np.abs(lam + 5.0)
    assert err[30] < err[10] * (0.6 ** 2) ** 15                             # (3/5)^2 per step, with slack
    lam0, _ = oracle.power_iteration(lambda x: 0.0 * x, r.standard_normal(n), 3)
    assert (lam0 == 0).all()


# ---- asymmetric group ranges given by the caller (App.: the range may be a sub-interval of [min, max]) ---------------
@pytest.mark.parametrize("bits", BITS)
def test_given_asymmetric_range_pins(bits):
    from fractions import Fraction
    L = 2 ** bits - 1
    rng = np.random.default_rng(70 + bits)
    # (a) lo = min, hi = max of every group reproduces the data-range quantizer bit for bit
    W = rng.normal(0.01, 0.05, (12, 64)).astype(np.float32)
    G = 3
    lo = W.reshape(G, -1).min(1)
    hi = W.reshape(G, -1).max(1)
    c0, d0, q0, r0 = oracle.quantize_groupwise_asym(W, bits, G)
    c1, d1, q1, r1 = oracle.quantize_groupwise_asym_range(W, bits, lo, hi)
    assert (c0 == c1).all() and (d0.view(np.uint32) == d1.view(np.uint32)).all() and (q0 == q1).all() and (r0 == r1).all()
    # (b) a lattice with exact arithmetic: lo = -3/8, Delta = 2^-4: codes = index, values below / above get 0 / L
    dlt = 2.0 ** -4
    lo1 = np.array([-0.375], np.float32)
    hi1 = np.array([-0.375 + L * dlt], np.float32)
    idx = rng.integers(0, L + 1, (4, 64))
    Wl = (-0.375 + dlt * idx).astype(np.float32)
    Wl[0, :4] = [-10.0, -0.376, hi1[0] + 1e-3, 99.0]
    c, d, q, r = oracle.quantize_groupwise_asym_range(Wl, bits, lo1, hi1)
    exp = idx.copy()
    exp[0, :4] = [0, 0, L, L]
    assert (c == exp).all() and d[0] == np.float32(dlt) and q[0] == np.float32(-0.375)
    assert (r == (exp - 2 ** (bits - 1)).sum(1)).all()
    # (c) nearest level of the clamped weight in exact rational arithmetic (away from ties by more than float error)
    lo2 = np.array([-0.11, 0.02], np.float32)
    hi2 = np.array([0.07, 0.09], np.float32)
    W2 = rng.normal(0.0, 0.08, (2, 256)).astype(np.float32)
    c, d, q, _ = oracle.quantize_groupwise_asym_range(W2, bits, lo2, hi2)
    for g in range(2):
        D, Q0, HI = Fraction(float(d[g])), Fraction(float(lo2[g])), Fraction(float(hi2[g]))
        for j in range(256):
            w = min(max(Fraction(float(W2[g, j])), Q0), HI)
            t = (w - Q0) / D
            near = min(max(int(round(t)), 0), L)
            if abs(t - near) < Fraction(4999, 10000):
                assert c[g, j] == near
            assert abs(int(c[g, j]) - t) <= Fraction(1, 2) + Fraction(1, 1000)
    # (d) a degenerate range lo == hi: Delta = 0, codes 0, Q = lo
    c, d, q, r = oracle.quantize_groupwise_asym_range(W2[:1], bits, np.array([0.05], np.float32), np.array([0.05], np.float32))
    assert (c == 0).all() and d[0] == 0.0 and (oracle.dequantize_groupwise_asym(c, d, q) == float(np.float32(0.05))).all()
    # (e) monotone in w, and a narrower range clips more weights to the end codes
    order = np.argsort(W2[0], kind="stable")
    cc, _, _, _ = oracle.quantize_groupwise_asym_range(W2[:1], bits, lo2[:1], hi2[:1])
    assert (np.diff(cc[0][order].astype(int)) >= 0).all()
    cn, _, _, _ = oracle.quantize_groupwise_asym_range(W2[:1], bits, lo2[:1] / 2, hi2[:1] / 2)
    assert ((cn == 0) | (cn == L)).sum() >= ((cc == 0) | (cc == L)).sum()


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_asymmetric_forward_with_per_token_scales(bits):
    """Asymmetric weights x per-token activation range: against the numpy fp64 product of the de-quantized operands
    (each row de-quantized with its own scale); a constant scale vector reproduces the fixed-clip asymmetric forward
    bit for bit; a row whose scale is doubled doubles exactly; an all-zero row (scale 0) gives exactly the bias."""
    T, N, K, G = 9, 12, 64, 4
    r = rng(140 + bits)
    W = (r.uniform(-0.02, 0.09, (N, K))).astype(np.float32)
    X = (r.standard_normal((T, K)) * r.uniform(0.1, 4.0, (T, 1))).astype(np.float32)
    X[4] = 0.0
    bias = r.standard_normal(N).astype(np.float32)
    codes, delta, q0, _ = oracle.quantize_groupwise_asym(W, bits, G)
    xq, rs_x, hx = oracle.quantize_act_dyn(X)
    What = oracle.dequantize_groupwise_asym(codes, delta, q0)
    Xhat = hx.astype(np.float64)[:, None] * (2.0 * xq.astype(np.float64) + 1.0)
    Y = oracle.qlinear_fwd_asym_dyn(xq, hx, codes, delta, q0)
    ref = Xhat @ What.T
    # the two terms Delta*S and q0*R may cancel: the bound is relative to their magnitudes
    R = (2 * xq.astype(np.int64) + 1).sum(axis=1)
    S = (2 * xq.astype(np.int64) + 1) @ codes.astype(np.int64).T
    rows = N // G
    mag = np.abs(hx.astype(np.float64))[:, None] * (np.abs(np.repeat(delta, rows).astype(np.float64))[None, :] * np.abs(S)
                                                     + np.abs(np.repeat(q0, rows).astype(np.float64))[None, :] * np.abs(R)[:, None])
    assert (np.abs(Y - ref) <= 1e-6 * mag + 1e-30).all()
    Yb = oracle.qlinear_fwd_asym_dyn(xq, hx, codes, delta, q0, bias=bias)
    assert (Yb[4] == bias).all() and (Y[4] == 0).all()
    # constant scales = the fixed clip
    xs, _ = oracle.quantize_act(X, 6.0)
    const = np.full(T, np.float32(6.0) / np.float32(255.0), np.float32)
    assert (oracle.qlinear_fwd_asym_dyn(xs, const, codes, delta, q0, bias=bias).view(np.uint32)
            == oracle.qlinear_fwd_asym(xs, 6.0, codes, delta, q0, bias=bias).view(np.uint32)).all()
    # a power of two on one row's scale
    hx2 = hx.copy()
    hx2[2] *= np.float32(2.0)
    Y2 = oracle.qlinear_fwd_asym_dyn(xq, hx2, codes, delta, q0)
    assert (Y2[2] == 2.0 * Y[2]).all() and (np.delete(Y2, 2, 0) == np.delete(Y, 2, 0)).all()
