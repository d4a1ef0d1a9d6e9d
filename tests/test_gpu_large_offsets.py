"""GPU: matrices with more than 2^31 elements, so that every row-times-pitch product in the kernels has to be a 64-bit
one: a 4.3 GB activation through the rotate+quantise kernel and a 4.4 GB output through the GEMM.  Rows are independent
in both (per-token scales), so the oracle checks a sample of rows, the last ones included, whose offsets lie past 2^31
elements (past 2^32 bytes).  The inputs are drawn on the device (seeded) because a host generator would take minutes."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import bf16_to_host_bits, check_codes, check_output, unpack_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cr():
    from paper_2512_03673_amd import binding
    binding.load()
    return binding


def sample_rows(M):
    return np.unique(np.concatenate([np.arange(0, 3), np.arange(M // 2 - 1, M // 2 + 2), np.arange(M - 37, M)]))


@pytest.mark.parametrize("g", (16, 256))
def test_rotquant_past_two_to_the_31_elements(cr, g):
    M, K = 66000, 32768                                   # 2.16e9 elements
    assert M * K > 2**31
    gen = torch.Generator(device="cuda").manual_seed(7 + g)
    X = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, M, 8192):                          # in slabs: randn has no bf16 path for 2^31 elements at once
        r1 = min(M, r0 + 8192)
        X[r0:r1] = torch.randn((r1 - r0, K), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    xq, xs = cr.convrot_rotquant_act(X, g)
    torch.cuda.synchronize()
    rows = sample_rows(M)
    codes = torch.empty((M, K), dtype=torch.int8, device="cuda")
    cr.convrot_unpack_codes(xq, M, K, codes)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    x_bits = X[idx].view(torch.int16).cpu().numpy().view(np.uint16)
    qo, so = oracle.rotquant(x_bits, g)
    check_codes(codes[idx].cpu().numpy(), xs[idx].cpu().numpy(), qo, so, f"rows past 2^31 elements, g={g}")
    # the layout itself, decoded on the host, for the last block of 32 rows (a whole number of blocks before it)
    first = (M // 32) * 32
    stages = -(-K // 128)
    tail = xq[first // 32 * stages * 3072:].cpu().numpy()
    last = unpack_host(tail, M - first, K)
    assert np.array_equal(last, codes[first:].cpu().numpy())


def test_gemm_output_past_two_to_the_31_elements(cr):
    M, N, K, g = 66000, 33000, 64, 16                     # Y: 2.18e9 elements
    assert M * N > 2**31
    gen = torch.Generator(device="cuda").manual_seed(11)
    X = torch.randn((M, K), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    W = (torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    bias = torch.randn((N,), generator=gen, device="cuda", dtype=torch.float32).mul_(0.1).to(torch.bfloat16)
    wq, ws = cr.convrot_prepare_weight(W, g)
    Y = cr.convlinear4bit_forward(X, wq, ws, g, bias=bias)
    torch.cuda.synchronize()
    rows = sample_rows(M)
    idx = torch.from_numpy(rows).cuda()
    x_bits = X[idx].view(torch.int16).cpu().numpy().view(np.uint16)
    w_bits = W.view(torch.int16).cpu().numpy().view(np.uint16)
    b_bits = bias.view(torch.int16).cpu().numpy().view(np.uint16)
    yo = oracle.convlinear4bit(x_bits, w_bits, g, bias=b_bits)
    check_output(bf16_to_host_bits(Y[idx]), yo, "rows of Y past 2^31 elements")
    # the integer product of the same rows, bit for bit, through the raw-accumulator entry point on the full problem
    xq, _ = cr.convrot_rotquant_act(X, g)
    acc = cr.convrot_w4a4_gemm_i32(xq, wq, M, N, K)
    torch.cuda.synchronize()
    cx = torch.empty((M, K), dtype=torch.int8, device="cuda")
    cr.convrot_unpack_codes(xq, M, K, cx)
    cw = torch.empty((N, K), dtype=torch.int8, device="cuda")
    cr.convrot_unpack_codes(wq, N, K, cw)
    torch.cuda.synchronize()
    want = oracle.int_gemm(cx[idx].cpu().numpy(), cw.cpu().numpy())
    assert np.array_equal(acc[idx].cpu().numpy(), want)
