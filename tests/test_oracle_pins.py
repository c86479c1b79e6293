"""Pins the C oracle (plain integer definition) to things other than itself:
the paper's method walked through literally (oracle/alg1.py, itself pinned to
Tables 1-2), brute force, closed forms, invariants, the conventional
decomposition of Eq. 2 written as third code, and library integer matmul /
convolution."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from oracle import alg1


def _dot_py(lw, la, act_mode):
    return sum((int(w) - 1) * (int(a) if act_mode else int(a) - 1) for w, a in zip(lw, la))


# --------------------------------------------------------------------------- Eq. 3 identity
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_eq3_identity_exhaustive_small_vectors(n):
    vecs = list(itertools.product(range(3), repeat=n))
    if n == 5:
        rnd = np.random.default_rng(0)
        vecs_y = [vecs[i] for i in rnd.choice(len(vecs), 40, replace=False)]
    else:
        vecs_y = vecs
    for x in vecs:
        for y in vecs_y:
            assert alg1.inner_product_levels(y, x, 0) == _dot_py(y, x, 0)


@pytest.mark.parametrize("n", [1, 2, 3])
def test_eq3_identity_over_all_codec_spellings(n):
    # every way of spelling the value 0 (01 or 10), in both operands
    for xc in itertools.product(range(4), repeat=n):
        for yc in itertools.product(range(4), repeat=n):
            want = sum(alg1.decode_field(a) * alg1.decode_field(b) for a, b in zip(xc, yc))
            assert alg1.inner_product_codecs(xc, yc) == want


def test_c_oracle_equals_method_as_printed_random_and_ragged():
    rnd = np.random.default_rng(11)
    for K in [1, 2, 3, 4, 5, 7, 8, 31, 32, 33, 63, 64, 65, 130]:
        Lw = rnd.integers(0, 3, size=(3, K), dtype=np.int8)
        La = rnd.integers(0, 3, size=(4, K), dtype=np.int8)
        for mode in (oracle.SYM, oracle.RELU):
            got = oracle.ternary_gemm(Lw, La, mode)
            want = alg1.gemm_levels(Lw, La, mode)
            assert np.array_equal(got, want), (K, mode)


def test_c_oracle_brute_force_tiny():
    for K in (1, 2, 3):
        vecs = np.array(list(itertools.product(range(3), repeat=K)), dtype=np.int8)
        for mode in (0, 1):
            C = oracle.ternary_gemm(vecs, vecs, mode)
            for i, w in enumerate(vecs):
                for j, a in enumerate(vecs):
                    assert C[i, j] == _dot_py(w, a, mode)


# --------------------------------------------------------------------------- closed forms / invariants
def test_closed_forms():
    K = 77
    two = np.full((2, K), 2, np.int8)
    zero = np.zeros((2, K), np.int8)
    one = np.ones((2, K), np.int8)
    assert (oracle.ternary_gemm(two, two, 0) == K).all()
    assert (oracle.ternary_gemm(two, zero, 0) == -K).all()
    assert (oracle.ternary_gemm(zero, zero, 0) == K).all()
    assert (oracle.ternary_gemm(one, two, 0) == 0).all()
    assert (oracle.ternary_gemm(two, one, 0) == 0).all()
    assert (oracle.ternary_gemm(two, two, 1) == 2 * K).all()
    assert (oracle.ternary_gemm(zero, two, 1) == -2 * K).all()
    assert (oracle.ternary_gemm(two, zero, 1) == 0).all()
    assert (oracle.ternary_gemm(two, one, 1) == K).all()


def test_invariants_random():
    rnd = np.random.default_rng(3)
    M, N, K = 9, 13, 203
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    C = oracle.ternary_gemm(Lw, La, 0)
    # negating the weights (level l -> 2-l, the bitwise complement of the codec) negates C
    assert np.array_equal(oracle.ternary_gemm((2 - Lw).astype(np.int8), La, 0), -C)
    # symmetric mode: swapping the operands transposes the result
    assert np.array_equal(oracle.ternary_gemm(La, Lw, 0), C.T)
    # parity and magnitude bounds
    nzw = (Lw != 1)
    nza = (La != 1)
    both = nzw.astype(np.int64) @ nza.astype(np.int64).T
    assert np.array_equal(C & 1, both & 1)
    assert (np.abs(C) <= both).all()
    # ReLU mode = symmetric mode + sum of the weights (second constraint)
    Cr = oracle.ternary_gemm(Lw, La, 1)
    wsum = (Lw.astype(np.int64) - 1).sum(axis=1)
    assert np.array_equal(Cr, C + wsum[:, None])
    # zero-weight padding of K changes nothing (ragged-tail reading)
    Lw2 = np.concatenate([Lw, np.ones((M, 53), np.int8)], axis=1)
    La2 = np.concatenate([La, rnd.integers(0, 3, size=(N, 53), dtype=np.int8)], axis=1)
    assert np.array_equal(oracle.ternary_gemm(Lw2, La2, 0), C)
    assert np.array_equal(oracle.ternary_gemm(Lw2, La2, 1), Cr)


def test_levels_outside_range_rejected():
    Lw = np.array([[0, 1, 3]], np.int8)
    La = np.array([[0, 1, 2]], np.int8)
    with pytest.raises(ValueError):
        oracle.ternary_gemm(Lw, La, 0)
    with pytest.raises(ValueError):
        oracle.ternary_gemm(La, np.array([[0, -1, 2]], np.int8), 0)


# --------------------------------------------------------------------------- library pins
@pytest.mark.parametrize("mode", [0, 1])
def test_c_oracle_vs_library_integer_matmul(mode):
    case = si.GemmCase("t", 96, 160, 1153, mode, config=9)
    Lw, La = case.make()
    C = oracle.ternary_gemm(Lw, La, mode)
    Vw = torch.from_numpy(Lw.astype(np.int64) - 1)
    Va = torch.from_numpy(La.astype(np.int64) - (0 if mode else 1))
    want = (Vw @ Va.T).numpy()
    assert np.array_equal(C, want)


def test_cfg1_statistics_and_library():
    case = si.cfg1()
    Lw, La = case.make()
    C = oracle.ternary_gemm(Lw, La, 0)
    want = (torch.from_numpy(Lw.astype(np.float32) - 1) @ torch.from_numpy(La.astype(np.float32) - 1).T).numpy()
    assert np.array_equal(C, want.astype(np.int32))     # fp32 exact: |partial sums| < 2^24
    # iid uniform levels: mean 0, variance K * (2/3)^2
    assert abs(C.mean()) < 0.5
    assert abs(C.var() / (case.K * 4 / 9) - 1) < 0.05


# --------------------------------------------------------------------------- convolution
def _conv_torch(Lw, Lx, stride, pad, mode):
    w = torch.from_numpy(Lw.astype(np.float64) - 1).permute(0, 3, 1, 2)          # OHWI -> OIHW
    x = torch.from_numpy(Lx.astype(np.float64) - (0 if mode else 1)).permute(0, 3, 1, 2)
    y = torch.nn.functional.conv2d(x, w, stride=stride, padding=pad)
    return y.permute(0, 2, 3, 1).numpy().astype(np.int64)


@pytest.mark.parametrize("R,stride,pad", [(3, 1, 1), (3, 2, 1), (1, 1, 0), (1, 2, 0)])
@pytest.mark.parametrize("mode", [0, 1])
def test_conv_vs_library(R, stride, pad, mode):
    rnd = np.random.default_rng(R * 10 + stride + mode)
    Lw = rnd.integers(0, 3, size=(5, R, R, 32), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(2, 9, 7, 32), dtype=np.int8)
    Y = oracle.ternary_conv2d(Lw, Lx, stride, pad, mode)
    assert np.array_equal(Y, _conv_torch(Lw, Lx, stride, pad, mode))


def _im2col(Lx, R, S, stride, pad, pad_level):
    B, H, W, C = Lx.shape
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    cols = np.full((B * Ho * Wo, R * S * C), pad_level, dtype=np.int8)
    n = 0
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for r in range(R):
                    for s in range(S):
                        hi, wi = ho * stride - pad + r, wo * stride - pad + s
                        if 0 <= hi < H and 0 <= wi < W:
                            cols[n, (r * S + s) * C:(r * S + s + 1) * C] = Lx[b, hi, wi]
                n += 1
    return cols


@pytest.mark.parametrize("mode", [0, 1])
def test_conv_equals_im2col_plus_gemm(mode):
    # Supplementary S1: conv = im2col + gemm.  The padded taps carry the level whose value is 0.
    rnd = np.random.default_rng(21 + mode)
    Lw = rnd.integers(0, 3, size=(6, 3, 3, 8), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(2, 6, 5, 8), dtype=np.int8)
    for stride in (1, 2):
        Y = oracle.ternary_conv2d(Lw, Lx, stride, 1, mode)
        cols = _im2col(Lx, 3, 3, stride, 1, pad_level=0 if mode else 1)
        C = oracle.ternary_gemm(Lw.reshape(6, -1), cols, mode)           # [Cout][pixels]
        assert np.array_equal(Y.reshape(-1, 6), C.T)


def test_conv_1x1_is_gemm_and_border_counts():
    rnd = np.random.default_rng(8)
    Lw = rnd.integers(0, 3, size=(7, 1, 1, 16), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(3, 4, 5, 16), dtype=np.int8)
    Y = oracle.ternary_conv2d(Lw, Lx, 1, 0, 0)
    C = oracle.ternary_gemm(Lw.reshape(7, 16), Lx.reshape(-1, 16), 0)
    assert np.array_equal(Y.reshape(-1, 7), C.T)
    # all-(+1) weights and activations: output = C * number of in-bounds taps (4C / 6C / 9C)
    Cc = 8
    Lw = np.full((1, 3, 3, Cc), 2, np.int8)
    Lx = np.full((1, 5, 5, Cc), 2, np.int8)
    Y = oracle.ternary_conv2d(Lw, Lx, 1, 1, 0)[0, :, :, 0]
    assert Y[0, 0] == 4 * Cc and Y[0, 2] == 6 * Cc and Y[2, 2] == 9 * Cc and Y[4, 4] == 4 * Cc
    # ReLU mode pads with the value 0 too: all level-2 activations (value 2)
    Y = oracle.ternary_conv2d(Lw, Lx, 1, 1, 1)[0, :, :, 0]
    assert Y[0, 0] == 8 * Cc and Y[2, 2] == 18 * Cc


# --------------------------------------------------------------------------- Eq. 2 (conventional 2-bit)
def _eq2_literal(Qw, Qa, alpha, beta):
    """Eq. 2 with the binary inner product of Eq. 1, written out plane by plane."""
    M, K = Qw.shape
    N = Qa.shape[0]
    out = np.zeros((M, N), dtype=np.float64)
    for m in range(2):
        xm = (Qw >> m) & 1
        for k in range(2):
            yk = (Qa >> k) & 1
            xnor_pop = K - (xm[:, None, :] ^ yk[None, :, :]).sum(axis=2)       # popcount(xnor)
            out += alpha[m] * beta[k] * (2 * xnor_pop - K)                     # Eq. 1
    return out


def test_twobit_oracle_vs_eq2_literal_and_bruteforce():
    rnd = np.random.default_rng(4)
    Qw = rnd.integers(0, 4, size=(5, 37), dtype=np.int8)
    Qa = rnd.integers(0, 4, size=(6, 37), dtype=np.int8)
    Cu = oracle.twobit_gemm(Qw, Qa, oracle.BASIS_UNIFORM)
    assert np.array_equal(Cu, _eq2_literal(Qw, Qa, (1, 2), (1, 2)).astype(np.int64))
    Ct = oracle.twobit_gemm(Qw, Qa, oracle.BASIS_TERNARY)
    assert np.array_equal(Ct, _eq2_literal(Qw, Qa, (0.5, 0.5), (0.5, 0.5)).astype(np.int64))
    # brute force: uniform basis values are 2q-3
    want = (2 * Qw.astype(np.int64) - 3) @ (2 * Qa.astype(np.int64) - 3).T
    assert np.array_equal(Cu, want)
    # all 16 code pairs, K = 1
    q = np.arange(4, dtype=np.int8).reshape(4, 1)
    tv = np.array([-1, 0, 0, 1])
    assert np.array_equal(oracle.twobit_gemm(q, q, oracle.BASIS_TERNARY), np.outer(tv, tv))


def test_twobit_on_ternary_codes_equals_ternary_oracle():
    # The codec of Table 1 is the two-plane {-1,+1} decomposition with alpha = (1/2, 1/2):
    # the conventional O(4N) evaluation of Eq. 2 and the O(2N) one of Eq. 3 must agree.
    rnd = np.random.default_rng(6)
    Lw = rnd.integers(0, 3, size=(8, 131), dtype=np.int8)
    La = rnd.integers(0, 3, size=(9, 131), dtype=np.int8)
    code = np.array([0, 1, 3], dtype=np.int8)
    code_alt = np.array([0, 2, 3], dtype=np.int8)
    C = oracle.ternary_gemm(Lw, La, 0)
    assert np.array_equal(oracle.twobit_gemm(code[Lw], code[La], oracle.BASIS_TERNARY), C)
    assert np.array_equal(oracle.twobit_gemm(code_alt[Lw], code[La], oracle.BASIS_TERNARY), C)


# --------------------------------------------------------------------------- scale epilogue
def test_scale_epilogue():
    rnd = np.random.default_rng(2)
    C = rnd.integers(-9000, 9000, size=(6, 11), dtype=np.int32)
    scale = rnd.uniform(0.5, 1.5, 6).astype(np.float32)
    bias = rnd.standard_normal(6).astype(np.float32)
    assert np.array_equal(C.astype(np.float32).astype(np.int64), C)        # float(C) exact
    got = oracle.scale_epilogue(C, scale, None, channel_is_row=True)
    assert np.array_equal(got, scale[:, None] * C.astype(np.float32))
    got = oracle.scale_epilogue(C, scale, bias, channel_is_row=True)
    assert np.array_equal(got, (scale[:, None] * C.astype(np.float32)) + bias[:, None])
    # NHWC: channel is the last axis
    Cn = rnd.integers(-500, 500, size=(2, 3, 4, 6), dtype=np.int32)
    got = oracle.scale_epilogue(Cn, scale, bias, channel_is_row=False)
    assert np.array_equal(got, scale * Cn.astype(np.float32) + bias)
    # against exact arithmetic: one multiply is correctly rounded
    exact = scale.astype(np.float64)[:, None] * C.astype(np.float64)
    assert np.array_equal(oracle.scale_epilogue(C, scale, None, True), exact.astype(np.float32))


# --------------------------------------------------------------------------- Eq. 1 and the xnor-only ablation
def test_binary_oracle_eq1():
    rnd = np.random.default_rng(31)
    K = 131
    Bw = rnd.integers(0, 2, size=(6, K), dtype=np.int8)
    Ba = rnd.integers(0, 2, size=(7, K), dtype=np.int8)
    C = oracle.binary_gemm(Bw, Ba)
    # Eq. 1 written with popcounts: 2 * popcount(xnor) - N
    xnor_pop = K - (Bw[:, None, :] ^ Ba[None, :, :]).sum(axis=2)
    assert np.array_equal(C, 2 * xnor_pop - K)
    assert (oracle.binary_gemm(Bw, Bw).diagonal() == K).all()
    assert (oracle.binary_gemm(Bw, (1 - Bw).astype(np.int8)).diagonal() == -K).all()
    with pytest.raises(ValueError):
        oracle.binary_gemm(np.array([[2]], np.int8), np.array([[1]], np.int8))


def test_xnor_only_is_wrong_exactly_where_both_operands_are_zero():
    # Table 2's bold rows: plain xnor fails only for 0 * 0.  With 0 spelled 01 in both operands the
    # error is +1 per such pair, so the ablated inner product = true product + #(both zero).
    rnd = np.random.default_rng(32)
    Lw = rnd.integers(0, 3, size=(5, 67), dtype=np.int8)
    La = rnd.integers(0, 3, size=(6, 67), dtype=np.int8)
    got = alg1.gemm_xnor_only(Lw, La)
    both_zero = (Lw == 1).astype(np.int64) @ (La == 1).astype(np.int64).T
    assert np.array_equal(got, oracle.ternary_gemm(Lw, La, 0) + both_zero)
    # per codec pair, against Table 2's value column
    for xc in range(4):
        for yc in range(4):
            true = alg1.decode_field(xc) * alg1.decode_field(yc)
            z = alg1.inner_product_xnor_only([xc], [yc])
            exception = alg1.decode_field(xc) == 0 and alg1.decode_field(yc) == 0
            assert (z != true) == exception
