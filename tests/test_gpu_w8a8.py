"""GPU parity of the W8A8 variant of the layer (8-bit codes on both operands) against the CPU oracle.

Gates as for the 4-bit path: codes identical on >= 99.99 % of elements and never more than 1 LSB apart,
int32 GEMM bit-exact on identical codes, bf16 output max relative error <= 1e-2 with cosine >= 0.9999.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import (bf16_to_host_bits, bf16_ulp_diff, bits_to_f64, check_output, codes8_to_dev, to_dev_bf16,
                      ulp_diff_f32, unpack_host8)
from paper_2512_03673_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cr():
    from paper_2512_03673_amd import binding
    binding.load()
    return binding


def check_codes8(q_gpu, s_gpu, q_ref, s_ref, what):
    d = np.abs(q_gpu.astype(np.int16) - q_ref.astype(np.int16))
    assert d.max(initial=0) <= 1, f"{what}: code off by {d.max()} LSB"
    frac = float((d == 0).mean()) if d.size else 1.0
    assert frac >= 0.9999, f"{what}: only {frac:.6%} identical"
    assert np.abs(q_gpu.astype(np.int16)).max(initial=0) <= 127, what
    assert ulp_diff_f32(s_gpu, s_ref).max(initial=0) <= 2, what
    return frac


@pytest.mark.parametrize("g", (4, 16, 64, 256, 1024))
@pytest.mark.parametrize("M,K", [(37, 1024), (5, 3072), (3, 12288), (2, 65536), (67, 2048), (19, 64), (19, 320)])
def test_rotquant8_matches_oracle(cr, g, M, K):
    if K % g:
        pytest.skip("K not a multiple of g")
    spec = wl.LayerSpec(f"rq8_{M}_{K}", M=M, K=K, N=8, group=g, x_col_count=max(1, K // 100), x_row_count=1, seed=13)
    x = wl.make_activation(spec)
    q, s = cr.convrot_rotquant_act8(to_dev_bf16(x), g)
    torch.cuda.synchronize()
    qo, so = oracle.rotquant(x, g, qmax=127)
    assert q.numel() == cr.packed_bytes8(M, K)
    frac = check_codes8(unpack_host8(q, M, K), s.cpu().numpy(), qo, so, f"g={g} M={M} K={K}")
    assert frac == 1.0


def test_rotquant8_closed_forms(cr):
    g, K = 16, 64
    x = np.zeros((4, K), dtype=np.float32)
    x[0, 37] = 1.0
    x[1, :] = -0.75
    x[3, 5] = -3.0
    bits = wl.f32_to_bf16_bits(x)
    q, s = cr.convrot_prepare_weight8(to_dev_bf16(bits), g)
    torch.cuda.synchronize()
    qo, so = oracle.rotquant(bits, g, qmax=127)
    q = unpack_host8(q, 4, K)
    assert np.array_equal(q, qo) and np.array_equal(s.cpu().numpy(), so)
    assert (q[1] == -127).all() and s[2].item() == 1.0 and not q[2].any()


@pytest.mark.parametrize("M,N,K", [(256, 128, 64), (300, 520, 1024), (1, 1, 64), (33, 7, 192), (257, 513, 3072), (35, 19, 96),
                                   (64, 1030, 12288), (513, 258, 128), (40, 136, 65536)])
def test_gemm8_i32_bit_exact(cr, M, N, K):
    rng = np.random.default_rng(M * 5 + N * 3 + K)
    qx = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    qw = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    qx[0, :] = 127
    qw[0, :] = -127           # reaches the accumulator bound 127^2 K
    acc = cr.convrot_w8a8_gemm_i32(codes8_to_dev(qx), codes8_to_dev(qw), M, N, K)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), oracle.int_gemm(qx, qw))


@pytest.mark.parametrize("M,N,K", [(3072, 3072, 64), (3001, 3067, 160), (3072, 3072, 3072), (3001, 3070, 1056),
                                   (3001, 3067, 256)])
def test_gemm8_on_square_tiles(cr, M, N, K):
    # The shapes above all take the 256 x 128 block tile (at most 256 tiles of either shape); these take the
    # 192 x 192 one, whole and with ragged edges: raw accumulators bit-exact, then the dequantising epilogue.
    # K = 64 and 160 stay inside the ring's prologue; K = 256, 1056 and 3072 are 4, 17 (the last one padded) and 48
    # stages of 64 codes, which run the steady-state loop that refills the ring.
    assert cr.gemm_tile_rows(M, N) == 192 and cr.gemm_tile_rows(300, 520) == 256
    rng = np.random.default_rng(M + N + K)
    qx = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    qw = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    qx[0, :] = 127
    qw[0, :] = -127
    xq, wq = codes8_to_dev(qx), codes8_to_dev(qw)
    ref = oracle.int_gemm(qx, qw)
    acc = cr.convrot_w8a8_gemm_i32(xq, wq, M, N, K)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref)
    sx = np.exp(rng.uniform(-6, 2, M)).astype(np.float32)
    sw = np.exp(rng.uniform(-9, -4, N)).astype(np.float32)
    bias = wl.f32_to_bf16_bits((rng.standard_normal(N) * 0.5).astype(np.float32))
    y = cr.convrot_w8a8_gemm_dequant(xq, torch.from_numpy(sx).cuda(), wq, torch.from_numpy(sw).cuda(), K)
    torch.cuda.synchronize()
    d = bf16_ulp_diff(bf16_to_host_bits(y), oracle.dequant(ref, sx, sw))
    assert d.max() <= 1 and (d == 0).mean() > 0.999
    y = cr.convrot_w8a8_gemm_dequant(xq, torch.from_numpy(sx).cuda(), wq, torch.from_numpy(sw).cuda(), K,
                                     bias=to_dev_bf16(bias))
    torch.cuda.synchronize()
    check_output(bf16_to_host_bits(y), oracle.dequant(ref, sx, sw, bias), "dequant8+bias, square tiles")


@pytest.mark.parametrize("M,N,K,with_bias", [(300, 520, 1024, False), (129, 1026, 3072, True), (31, 5, 64, True)])
def test_gemm8_dequant_on_identical_codes(cr, M, N, K, with_bias):
    rng = np.random.default_rng(M + N + K)
    qx = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    qw = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    sx = np.exp(rng.uniform(-6, 2, M)).astype(np.float32)
    sw = np.exp(rng.uniform(-9, -4, N)).astype(np.float32)
    bias = wl.f32_to_bf16_bits((rng.standard_normal(N) * 0.5).astype(np.float32)) if with_bias else None
    y = cr.convrot_w8a8_gemm_dequant(codes8_to_dev(qx), torch.from_numpy(sx).cuda(), codes8_to_dev(qw),
                                     torch.from_numpy(sw).cuda(), K, bias=None if bias is None else to_dev_bf16(bias))
    torch.cuda.synchronize()
    yb = bf16_to_host_bits(y)
    yo = oracle.dequant(oracle.int_gemm(qx, qw), sx, sw, bias)
    if bias is None:
        d = bf16_ulp_diff(yb, yo)
        assert d.max() <= 1 and (d == 0).mean() > 0.999
    check_output(yb, yo, "dequant8")


@pytest.mark.parametrize("g", (16, 256))
def test_forward8_tiny_config(cr, g):
    base = wl.CONFIGS["cfg1_tiny"][0]
    spec = wl.LayerSpec(**{**base.__dict__, "group": g})
    x, w = wl.make_layer(spec)
    bias = wl.make_bias(spec)
    wq, ws = cr.convrot_prepare_weight8(to_dev_bf16(w), g)
    y = cr.convlinear8bit_forward(to_dev_bf16(x), wq, ws, g, bias=to_dev_bf16(bias))
    xq, xs = cr.convrot_rotquant_act8(to_dev_bf16(x), g)
    y2 = cr.convrot_w8a8_gemm_dequant(xq, xs, wq, ws, spec.K, bias=to_dev_bf16(bias))
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    yo = oracle.convlinear(x, w, g, bias=bias, qmax=127)
    rel, cos = check_output(bf16_to_host_bits(y), yo, f"forward8 g={g}")
    # and it is closer to the unquantised product than the 4-bit layer is
    ref = bits_to_f64(x) @ bits_to_f64(w).T + bits_to_f64(bias)[None, :]
    e8 = np.linalg.norm(bits_to_f64(bf16_to_host_bits(y)) - ref)
    e4 = np.linalg.norm(bits_to_f64(oracle.convlinear(x, w, g, bias=bias, qmax=7)) - ref)
    assert e8 < e4 / 4


def test_forward8_full_size_headline_shape(cr):
    spec = wl.HEADLINE
    print(f"case w8a8 {spec.name}: M={spec.M} K={spec.K} N={spec.N}", flush=True)
    x, w = wl.make_layer(spec)
    wq, ws = cr.convrot_prepare_weight8(to_dev_bf16(w), spec.group)
    y = cr.convlinear8bit_forward(to_dev_bf16(x), wq, ws, spec.group)
    xq, xs = cr.convrot_rotquant_act8(to_dev_bf16(x), spec.group)
    torch.cuda.synchronize()
    qwo, swo = oracle.rotquant(w, spec.group, qmax=127)
    qxo, sxo = oracle.rotquant(x, spec.group, qmax=127)
    assert check_codes8(unpack_host8(wq, spec.N, spec.K), ws.cpu().numpy(), qwo, swo, "W8") == 1.0
    assert check_codes8(unpack_host8(xq, spec.M, spec.K), xs.cpu().numpy(), qxo, sxo, "X8") == 1.0
    rows = np.array(sorted(set([0, 255, 256, spec.M - 1]) | set(np.random.default_rng(0).choice(spec.M, 24, replace=False).tolist())))
    rt = torch.from_numpy(rows).cuda()
    acc = cr.convrot_w8a8_gemm_i32(codes8_to_dev(qxo[rows]), wq, len(rows), spec.N, spec.K)
    torch.cuda.synchronize()
    acc_o = oracle.int_gemm(qxo[rows], qwo)
    assert np.array_equal(acc.cpu().numpy(), acc_o)
    yo = oracle.dequant(acc_o, sxo[rows], swo)
    d = bf16_ulp_diff(bf16_to_host_bits(y[rt]), yo)
    assert d.max() <= 1
    check_output(bf16_to_host_bits(y[rt]), yo, "forward8 headline")


def test_w8a8_k_multiple_of_32_with_zero_padded_last_stage(cr):
    # K = 96: one and a half 64-byte stages per row; the layout pads the second with zero codes
    spec = wl.LayerSpec("w8_k96", M=35, K=96, N=19, group=16, seed=21)
    x, w = wl.make_layer(spec)
    wq, ws = cr.convrot_prepare_weight8(to_dev_bf16(w), 16)
    y = cr.convlinear8bit_forward(to_dev_bf16(x), wq, ws, 16)
    torch.cuda.synchronize()
    check_output(bf16_to_host_bits(y), oracle.convlinear(x, w, 16, qmax=127), "forward8 K=96")
    x48 = torch.zeros((4, 48), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(cr.ConvRotError) as e:
        cr.convrot_rotquant_act8(x48, 16)
    assert e.value.status == -2
