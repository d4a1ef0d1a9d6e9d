"""Pins for the CPU oracle: what the paper and the mathematics fix, not the oracle itself.

Every check compares an oracle function with something that is *not* the oracle:
the matrix the paper prints (Thm 3.3, Eq. 9), the Hadamard identities of Sec. 3.2,
closed forms of the rotation and the quantiser on hand-made inputs, numpy library
routines with a different definition (np.kron, dense block-diagonal matmul, int64
matmul, X @ W.T) and the quantiser's own error bound.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2512_03673_amd import workloads as wl

GROUPS = (4, 16, 64, 256)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def as_f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


# ----------------------------------------------------------------------------- H_g
def test_h4_is_the_printed_matrix():
    printed = np.loadtxt(os.path.join(GOLDEN, "h4_regular_hadamard.txt"), dtype=np.int64)
    assert printed.shape == (4, 4)
    assert np.array_equal(oracle.hadamard(4).astype(np.int64), printed)


@pytest.mark.parametrize("g", GROUPS + (1024,))
def test_hadamard_identities(g):
    H = oracle.hadamard(g).astype(np.int64)
    root = int(round(np.sqrt(g)))
    assert set(np.unique(H)) == {-1, 1}
    # Def. of a Hadamard matrix (Eq. 3)
    assert np.array_equal(H @ H.T, g * np.eye(g, dtype=np.int64))
    # regular (Def. in Sec. 3.2): every row and column sums to +-sqrt(g); for this base all are +
    assert np.array_equal(H.sum(axis=0), np.full(g, root))
    assert np.array_equal(H.sum(axis=1), np.full(g, root))
    # column-sum-squared property (Thm 3.1, Eq. 4) and minimal column discrepancy (Thm 3.2, Eq. 8)
    assert int((H.sum(axis=0) ** 2).sum()) == g * g
    assert int(np.abs(H.sum(axis=0)).max()) == root
    # symmetric => the normalised matrix is an involution
    assert np.array_equal(H, H.T)


@pytest.mark.parametrize("g", (16, 64, 256))
def test_kronecker_recursion_matches_numpy_kron(g):
    H4 = oracle.hadamard(4).astype(np.int64)
    assert np.array_equal(oracle.hadamard(g).astype(np.int64), np.kron(oracle.hadamard(g // 4).astype(np.int64), H4))


def test_sylvester_is_not_regular_negative_control():
    # Sec. 3.2: the Sylvester matrix has an all-ones column, discrepancy n (Eq. 7 upper bound)
    S = np.array([[1]])
    for _ in range(4):
        S = np.block([[S, S], [S, -S]])
    assert np.abs(S.sum(axis=0)).max() == 16
    assert np.abs(oracle.hadamard(16).astype(int).sum(axis=0)).max() == 4


def test_other_base_j_minus_2i_is_group_reversal():
    # J - 2I equals the printed matrix with its columns reversed; Kronecker powers keep that
    # relation (reversal of the whole group), so rotated values are the same set, mirrored.
    base = np.ones((4, 4), dtype=np.int8) - 2 * np.eye(4, dtype=np.int8)
    for g in GROUPS:
        Hp = oracle.hadamard(g)
        Hj = oracle.hadamard(g, base)
        assert np.array_equal(Hj[:, ::-1], Hp)


# ----------------------------------------------------------------------------- rotation
@pytest.mark.parametrize("g", GROUPS)
def test_rotation_closed_forms(g):
    K = 2 * g if g >= 16 else 32
    root = np.sqrt(g)
    H = oracle.hadamard(g).astype(np.float64)
    # constant block c*1 -> c*1 (1^T H = sqrt(g) 1^T): a one-signed row is not concentrated
    x = np.full((1, K), 3.0, dtype=np.float32)
    assert np.array_equal(oracle.rotate(bf16(x), g), np.full((1, K), 3.0))
    # one-hot e_j inside block b -> row j of H / sqrt(g), other blocks stay zero
    for j in (0, 1, g - 1, g // 2 + 1):
        x = np.zeros((1, K), dtype=np.float32)
        x[0, g + j] = 2.0
        out = oracle.rotate(bf16(x), g)
        assert np.array_equal(out[0, g:2 * g], 2.0 * H[j] / root)
        assert not out[0, :g].any() and not out[0, 2 * g:].any()


@pytest.mark.parametrize("g", GROUPS)
def test_rotation_matches_dense_block_diagonal_matmul(g):
    rng = np.random.default_rng(g)
    K = 3 * g if g >= 16 else 48
    x = bf16(rng.standard_normal((5, K)))
    H = oracle.hadamard(g).astype(np.float64) / np.sqrt(g)
    B = np.zeros((K, K))
    for b in range(K // g):
        B[b * g:(b + 1) * g, b * g:(b + 1) * g] = H
    want = as_f64(x) @ B
    got = oracle.rotate(x, g)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    # orthogonality: energy is preserved, twice is the identity
    np.testing.assert_allclose((got ** 2).sum(axis=1), (as_f64(x) ** 2).sum(axis=1), rtol=1e-13)
    np.testing.assert_allclose(got @ B, as_f64(x), rtol=0, atol=1e-13)


@pytest.mark.parametrize("g", GROUPS)
def test_rotation_invariance_of_the_product(g):
    # Eq. 2 / Eq. 13: sum_i RHT(X_i) RHT(W_i)^T = X W^T before quantisation
    rng = np.random.default_rng(100 + g)
    K = 512
    x = bf16(rng.standard_normal((7, K)) * 3)
    w = bf16(rng.standard_normal((9, K)) * 0.02)
    want = as_f64(x) @ as_f64(w).T
    got = oracle.rotate(x, g) @ oracle.rotate(w, g).T
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12 * np.abs(want).max() * K)


def test_rotation_rejects_ragged_k():
    with pytest.raises(ValueError):
        oracle.rotate(np.zeros((1, 24), dtype=np.uint16), 16)


def test_row_outlier_behaviour_regular_vs_sylvester():
    # Sec. 4.1 motivation: a one-signed (row-outlier) token is concentrated by the Sylvester
    # matrix (first column all ones) and left alone by the regular one.
    g, K = 64, 256
    x = np.full((1, K), 5.0, dtype=np.float32)
    S = np.array([[1.0]])
    for _ in range(6):
        S = np.block([[S, S], [S, -S]])
    syl = (x.reshape(-1, g) @ S / np.sqrt(g)).reshape(1, K)
    assert np.abs(syl).max() == 5.0 * np.sqrt(g)
    assert np.abs(oracle.rotate(bf16(x), g)).max() == 5.0


# ----------------------------------------------------------------------------- quantiser
def test_quantizer_ties_round_half_to_even_and_clamp():
    # scale = 7/7 = 1, so v/s = v: ties must go to the even neighbour
    v = np.array([[7.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, -6.5, 6.5, 0.49999, -0.50001]])
    codes, scale = oracle.quantize(v)
    assert scale[0] == np.float32(1.0)
    assert codes[0].tolist() == [7, 0, 2, 2, 4, 0, -2, -2, -6, 6, 0, -1]


def test_quantizer_zero_row_and_range():
    v = np.zeros((2, 8))
    v[1] = [-3, 1, 2, 3, -1, 0.2, 0, 0]
    codes, scale = oracle.quantize(v)
    assert scale[0] == np.float32(1.0) and not codes[0].any()
    assert scale[1] == np.float32(3.0 / 7.0)
    assert codes[1, 0] == -7 and codes.min() >= -7 and codes.max() <= 7


@pytest.mark.parametrize("g", GROUPS)
def test_quantizer_closed_forms_after_rotation(g):
    K = 4 * g
    H = oracle.hadamard(g).astype(np.int64)
    # one-hot row: rotated block = H[j]/sqrt(g) => codes = 7*H[j], scale = 1/(7 sqrt g)
    j = g - 2
    x = np.zeros((1, K), dtype=np.float32)
    x[0, 2 * g + j] = 1.0
    codes, scale = oracle.rotquant(bf16(x), g)
    assert np.array_equal(codes[0, 2 * g:3 * g].astype(np.int64), 7 * H[j])
    assert not codes[0, :2 * g].any() and not codes[0, 3 * g:].any()
    assert scale[0] == np.float32(1.0 / (7.0 * np.sqrt(g)))
    # constant row c: all codes 7*sign(c), scale |c|/7
    x = np.full((1, K), -0.75, dtype=np.float32)
    codes, scale = oracle.rotquant(bf16(x), g)
    assert np.array_equal(codes, np.full((1, K), -7, dtype=np.int8))
    assert scale[0] == np.float32(0.75 / 7.0)


@pytest.mark.parametrize("g", GROUPS)
def test_quantizer_error_bound_and_full_range(g):
    spec = wl.LayerSpec("pin", M=64, K=1024, N=8, group=g, seed=3)
    x = wl.make_activation(spec)
    rot = oracle.rotate(x, g)
    codes, scale = oracle.rotquant(x, g)
    s = scale.astype(np.float64)[:, None]
    err = np.abs(rot - codes.astype(np.float64) * s)
    # |x' - q s| <= s/2 (plus the fp32 rounding of s acting on |q| <= 7)
    assert (err <= 0.5 * s * (1 + 1e-6)).all()
    assert (np.abs(codes).max(axis=1) == 7).all()
    # the scale is absmax/7 rounded to fp32
    want = (np.abs(rot).max(axis=1) / 7.0).astype(np.float32)
    assert np.array_equal(scale, want)


def test_pack_layout_and_roundtrip():
    codes = np.array([[-7, 7, 0, -1, 3, -4, 1, 2]], dtype=np.int8)
    packed = oracle.pack4(codes)
    # byte j: code 2j in bits 0-3, code 2j+1 in bits 4-7, two's complement nibbles
    assert packed[0].tolist() == [0x79, 0xF0, 0xC3, 0x21]
    rng = np.random.default_rng(0)
    c = rng.integers(-7, 8, size=(5, 64)).astype(np.int8)
    assert np.array_equal(oracle.unpack4(oracle.pack4(c)), c)


# ----------------------------------------------------------------------------- integer GEMM
def test_int_gemm_matches_numpy_int64():
    rng = np.random.default_rng(1)
    qx = rng.integers(-7, 8, size=(13, 96)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(11, 96)).astype(np.int8)
    want = qx.astype(np.int64) @ qw.astype(np.int64).T
    got = oracle.int_gemm(qx, qw)
    assert got.dtype == np.int32 and got.shape == (13, 11)
    assert np.array_equal(got.astype(np.int64), want)
    # extreme codes reach the bound 49 K exactly
    K = 12288
    a = np.full((1, K), -7, dtype=np.int8)
    b = np.full((2, K), 7, dtype=np.int8)
    b[1] = -7
    assert oracle.int_gemm(a, b).tolist() == [[-49 * K, 49 * K]]


# ----------------------------------------------------------------------------- dequant / bf16
def test_bf16_rounding_matches_torch_and_ties():
    rng = np.random.default_rng(2)
    v = (rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096))).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.double_to_bf16(float(t)) for t in v], dtype=np.uint16)
    assert np.array_equal(got, want)
    # ties to even at 8 significant bits; double rounding through fp32 would get the third wrong
    assert oracle.double_to_bf16(1.0 + 2.0 ** -8) == 0x3F80          # tie -> even (1.0)
    assert oracle.double_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82      # tie -> even (1 + 2^-6)
    assert oracle.double_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert oracle.double_to_bf16(-0.0) == 0x8000
    assert oracle.double_to_bf16(3.5e38) == 0x7F80


def test_dequant_is_acc_times_both_scales():
    acc = np.array([[3, -5], [0, 150528]], dtype=np.int32)
    sx = np.array([0.5, 2.0 ** -10], dtype=np.float32)
    sw = np.array([0.25, 3.0], dtype=np.float32)
    y = as_f64(oracle.dequant(acc, sx, sw))
    # 150528*3/1024 = 441 needs 9 significant bits: a tie between 440 and 442, even is 440
    want = np.array([[0.375, -7.5], [0.0, 440.0]])
    assert np.array_equal(y, want)


# ----------------------------------------------------------------------------- whole forward
@pytest.mark.parametrize("g", GROUPS)
def test_forward_exact_when_rotated_operands_are_representable(g):
    # X rows constant, W rows one-hot: both rotate onto the 4-bit grid, so Y = X W^T exactly
    K, M, N = 4 * g, 3, 5
    x = np.zeros((M, K), dtype=np.float32)
    x[0], x[1], x[2] = 1.0, -2.0, 0.5
    w = np.zeros((N, K), dtype=np.float32)
    for n in range(N):
        w[n, (n * 7) % K] = 0.25 * (n + 1)
    y = as_f64(oracle.convlinear4bit(bf16(x), bf16(w), g))
    assert np.array_equal(y, x.astype(np.float64) @ w.astype(np.float64).T)


def test_forward_composition_and_error_budget():
    spec = wl.LayerSpec("pin_fwd", M=48, K=512, N=40, group=16, x_col_count=0, x_row_count=0, seed=5)
    x, w = wl.make_layer(spec)
    y = as_f64(oracle.convlinear4bit(x, w, 16))
    ref = as_f64(x) @ as_f64(w).T
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    # two independent 4-bit quantisers on near-Gaussian rotated data: roughly 10-20 % relative error
    assert 0.02 < rel < 0.3
    # stepwise composition gives the same bits as the one-call forward
    qx, sx = oracle.rotquant(x, 16)
    qw, sw = oracle.rotquant(w, 16)
    assert np.array_equal(oracle.dequant(oracle.int_gemm(qx, qw), sx, sw), oracle.convlinear4bit(x, w, 16))
    # analytic bound: |Y - X W^T| <= sum_k (|x'| sw/2 + |w'| sx/2 + sx sw/4) per element
    rx, rw = oracle.rotate(x, 16), oracle.rotate(w, 16)
    bound = (np.abs(rx).sum(1)[:, None] * sw[None, :] / 2 + np.abs(rw).sum(1)[None, :] * sx[:, None] / 2
             + spec.K * sx[:, None] * sw[None, :] / 4)
    assert (np.abs(y - ref) <= bound * 1.01 + np.abs(ref) * 2.0 ** -8).all()


def test_outliers_hurt_and_rotation_helps():
    base = dict(M=64, K=1024, N=64, group=16, seed=7)
    clean = wl.LayerSpec("pin_clean", x_col_count=0, x_row_count=0, **base)
    dirty = wl.LayerSpec("pin_clean", x_col_count=8, x_col_range=(50.0, 50.0), x_row_count=0, **base)

    def rel_err(spec, g):
        x, w = wl.make_layer(spec)
        y = as_f64(oracle.convlinear4bit(x, w, g))
        ref = as_f64(x) @ as_f64(w).T
        return np.linalg.norm(y - ref) / np.linalg.norm(ref)

    assert rel_err(clean, 16) < rel_err(dirty, 16)
    # larger groups spread a channel outlier over more channels (Sec. 4.2)
    assert rel_err(dirty, 256) < rel_err(dirty, 16) < rel_err(dirty, 4)


# ----------------------------------------------------------------------------- bias and the W8A8 variant
def test_dequant_bias_is_added_before_the_single_rounding():
    acc = np.array([[3, -5], [0, 256]], dtype=np.int32)
    sx = np.array([0.5, 2.0 ** -8], dtype=np.float32)
    sw = np.array([0.25, 1.0], dtype=np.float32)
    bias = bf16([1.0, 2.0 ** -8])
    y = as_f64(oracle.dequant(acc, sx, sw, bias))
    # [1,1]: 256 * 2^-8 * 1 + 2^-8 = 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); rounding the
    # product (1.0) and the sum separately could not tell, rounding the exact sum once does
    # [0,1]: -2.5 + 2^-8 lies a quarter step (2^-6 in [2, 4)) from -2.5
    assert np.array_equal(y, np.array([[1.375, -2.5], [1.0, 1.0]]))
    # zero accumulators: the output is the bias itself; no bias: unchanged from the plain form
    z = np.zeros((2, 2), dtype=np.int32)
    assert np.array_equal(oracle.dequant(z, sx, sw, bias), np.tile(bias, (2, 1)))
    assert np.array_equal(oracle.dequant(acc, sx, sw, None), oracle.dequant(acc, sx, sw))


def test_forward_with_bias_on_representable_operands():
    g, K, M, N = 16, 64, 3, 5
    x = np.zeros((M, K), dtype=np.float32)
    x[0], x[1], x[2] = 1.0, -2.0, 0.5
    w = np.zeros((N, K), dtype=np.float32)
    for n in range(N):
        w[n, (n * 7) % K] = 0.25 * (n + 1)
    # (no exact cancellation against the bias: the fp32 scales make acc * s_x * s_w exact only to ~2^-24)
    b = np.array([0.75, -1.0, 0.0, 8.0, -0.125], dtype=np.float32)
    y = as_f64(oracle.convlinear4bit(bf16(x), bf16(w), g, bias=bf16(b)))
    assert np.array_equal(y, x.astype(np.float64) @ w.astype(np.float64).T + b[None, :])


def test_eight_bit_quantiser_closed_forms_and_bound():
    # same quantiser, 127 levels: one-hot row -> 127 * H[j] / ... only when sqrt(g) divides; use constant row
    x = np.full((1, 64), -0.75, dtype=np.float32)
    q, s = oracle.rotquant(bf16(x), 16, qmax=127)
    assert (q == -127).all() and s[0] == np.float32(0.75 / 127)
    rng = np.random.default_rng(3)
    v = rng.standard_normal((7, 256))
    q, s = oracle.quantize(v, qmax=127)
    assert np.abs(q.astype(int)).max(axis=1).tolist() == [127] * 7
    assert (np.abs(v - q * s[:, None].astype(np.float64)) <= s[:, None] / 2 * (1 + 1e-6)).all()
    assert np.array_equal(s, (np.abs(v).max(axis=1) / 127).astype(np.float32))
    # ties to even at 8 bits as at 4
    t = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -126.5]])
    q, s = oracle.quantize(t, qmax=127)
    assert s[0] == 1.0 and q[0].tolist() == [127, 0, 2, 2, 0, -2, -126]


def test_w8a8_forward_is_far_more_accurate_than_w4a4():
    spec = wl.LayerSpec("pin_w8", M=32, K=512, N=24, group=16, x_col_count=0, x_row_count=0, seed=9)
    x, w = wl.make_layer(spec)
    ref = as_f64(x) @ as_f64(w).T
    e4 = np.linalg.norm(as_f64(oracle.convlinear(x, w, 16, qmax=7)) - ref) / np.linalg.norm(ref)
    e8 = np.linalg.norm(as_f64(oracle.convlinear(x, w, 16, qmax=127)) - ref) / np.linalg.norm(ref)
    # uniform quantisation noise scales with the step: 127 / 7 = 18x finer
    assert e8 < e4 / 8 and e8 < 0.02
    qx, sx = oracle.rotquant(x, 16, qmax=127)
    qw, sw = oracle.rotquant(w, 16, qmax=127)
    assert np.array_equal(oracle.dequant(oracle.int_gemm(qx, qw), sx, sw), oracle.convlinear(x, w, 16, qmax=127))
    assert np.array_equal(oracle.int_gemm(qx, qw), qx.astype(np.int64) @ qw.astype(np.int64).T)
