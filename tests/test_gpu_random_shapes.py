"""GPU parity on seeded random small shapes: ragged M and N around the 192-row tile edges, every K % 32 == 0
residue of the 128-code stage, every group size that divides K, with and without a bias.  CONVROT_FUZZ_CASES in the
environment raises the number of cases (default 24 four-bit and 12 eight-bit ones) for a longer run."""
import os

import numpy as np
import pytest
import torch

import oracle
from gpu_util import bf16_to_host_bits, check_codes, check_output, to_dev_bf16, unpack_host, unpack_host8
from paper_2512_03673_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cr():
    from paper_2512_03673_amd import binding
    binding.load()
    return binding


def test_forward_on_random_shapes(cr):
    rng = np.random.default_rng(2024)
    for case in range(int(os.environ.get("CONVROT_FUZZ_CASES", 24))):
        M = int(rng.integers(1, 450))
        N = int(rng.integers(1, 450))
        K = 32 * int(rng.integers(1, 40))
        groups = [g for g in (4, 16, 64, 256, 1024) if K % g == 0]
        g = int(groups[rng.integers(len(groups))])
        with_bias = bool(rng.integers(2))
        print(f"case {case}: M={M} N={N} K={K} g={g} bias={with_bias}", flush=True)
        spec = wl.LayerSpec(f"rnd{case}", M=M, K=K, N=N, group=g, x_col_count=max(1, K // 100), x_row_count=1, seed=100 + case)
        x, w = wl.make_layer(spec)
        bias = wl.make_bias(spec) if with_bias else None
        wq, ws = cr.convrot_prepare_weight(to_dev_bf16(w), g)
        xq, xs = cr.convrot_rotquant_act(to_dev_bf16(x), g)
        y = cr.convlinear4bit_forward(to_dev_bf16(x), wq, ws, g, bias=None if bias is None else to_dev_bf16(bias))
        torch.cuda.synchronize()
        qxo, sxo = oracle.rotquant(x, g)
        qwo, swo = oracle.rotquant(w, g)
        check_codes(unpack_host(xq, M, K), xs.cpu().numpy(), qxo, sxo, f"case {case} X")
        check_codes(unpack_host(wq, N, K), ws.cpu().numpy(), qwo, swo, f"case {case} W")
        acc = cr.convrot_w4a4_gemm_i32(xq, wq, M, N, K)
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy(), oracle.int_gemm(unpack_host(xq, M, K), unpack_host(wq, N, K))), f"case {case}"
        check_output(bf16_to_host_bits(y), oracle.convlinear4bit(x, w, g, bias=bias), f"case {case}")


def test_forward8_on_random_shapes(cr):
    rng = np.random.default_rng(2025)
    for case in range(int(os.environ.get("CONVROT_FUZZ_CASES", 12))):
        M = int(rng.integers(1, 450))
        N = int(rng.integers(1, 450))
        K = 32 * int(rng.integers(1, 40))
        groups = [g for g in (4, 16, 64, 256, 1024) if K % g == 0]
        g = int(groups[rng.integers(len(groups))])
        with_bias = bool(rng.integers(2))
        print(f"case {case}: M={M} N={N} K={K} g={g} bias={with_bias}", flush=True)
        spec = wl.LayerSpec(f"rnd8_{case}", M=M, K=K, N=N, group=g, x_col_count=max(1, K // 100), x_row_count=1, seed=300 + case)
        x, w = wl.make_layer(spec)
        bias = wl.make_bias(spec) if with_bias else None
        wq, ws = cr.convrot_prepare_weight8(to_dev_bf16(w), g)
        xq, xs = cr.convrot_rotquant_act8(to_dev_bf16(x), g)
        y = cr.convlinear8bit_forward(to_dev_bf16(x), wq, ws, g, bias=None if bias is None else to_dev_bf16(bias))
        acc = cr.convrot_w8a8_gemm_i32(xq, wq, M, N, K)
        torch.cuda.synchronize()
        cx, cw = unpack_host8(xq, M, K), unpack_host8(wq, N, K)
        for c, bits, what in ((cx, x, "X"), (cw, w, "W")):
            qo, _ = oracle.rotquant(bits, g, qmax=127)
            d = np.abs(c.astype(np.int16) - qo.astype(np.int16))
            assert d.max() <= 1 and (d == 0).mean() >= 0.9999, f"case {case} {what}: {int((d != 0).sum())} codes differ, max {int(d.max())}"
        assert np.array_equal(acc.cpu().numpy(), oracle.int_gemm(cx, cw)), f"case {case}"
        check_output(bf16_to_host_bits(y), oracle.convlinear(x, w, g, bias=bias, qmax=127), f"case {case}")
