"""GPU parity at the full benchmark sizes (configurations 2-5), in the launch configuration bench.py times.

  * codes and scales of X and of W are compared in full;
  * the integer GEMM is launched on the whole [M, N] problem, on the code matrices kernel A left in
    HBM, so that the kernel instantiation and grid under test are the ones the benchmark times;
  * for M = 4608 (configurations 2-4 and the fused-width layer) the oracle computes the whole integer
    product and the whole bf16 output (a few seconds on the machine's host cores) and every element is compared;
  * for M = 16896 (configuration 5) the oracle computes a seeded sample of token rows, every output channel of
    each, which includes the rows on both sides of every tile boundary the kernels have;
  * properties that hold at any size cover the rest: every code in [-7, 7], every non-zero row
    reaches |7|, scales positive and finite, output finite.
Gates are the same as for the small cases (see gpu_util).
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import bf16_to_host_bits, bf16_ulp_diff, check_codes, check_output, to_dev_bf16, unpack_host
from paper_2512_03673_amd import workloads as wl

pytestmark = pytest.mark.gpu

FULL = [spec for cfg in ("cfg2_qkv", "cfg3_mlp", "cfg4_group_sweep", "cfg5_hires") for spec in wl.CONFIGS[cfg]]
FULL += list(wl.NEXT_CONFIGS["n1_fused_width"]) + list(wl.NEXT_CONFIGS["n3_group_1024"])    # run with a bias
WITH_BIAS = {"fused_out", "fused_out_g1024"}


@pytest.fixture(scope="module")
def cr():
    from paper_2512_03673_amd import binding
    binding.load()
    return binding


def sample_rows(M: int, seed: int, count: int = 40) -> np.ndarray:
    """Seeded rows plus the rows on both sides of every kind of tile boundary the kernels have."""
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 31, 32, 127, 128, 191, 192, 193, 255, 256, 257, 383, 384, M // 2, M - 257, M - 256, M - 193,
             M - 192, M - 191, M - 2, M - 1]
    rows = set(int(r) for r in fixed if 0 <= r < M)
    rows.update(int(r) for r in rng.choice(M, size=count, replace=False))
    return np.array(sorted(rows), dtype=np.int64)


@pytest.mark.parametrize("spec", FULL, ids=[s.name for s in FULL])
def test_full_size_layer(cr, spec):
    print(f"case {spec.name}: M={spec.M} K={spec.K} N={spec.N} g={spec.group}", flush=True)
    g = spec.group
    x, w = wl.make_layer(spec)

    # ---- HIP path, as bench.py runs it: offline weight prep, then the fused forward
    xd = to_dev_bf16(x)
    wq, ws = cr.convrot_prepare_weight(to_dev_bf16(w), g)
    ws_buf = torch.empty((cr.workspace_bytes(spec.M, spec.K),), dtype=torch.uint8, device="cuda")
    y = torch.empty((spec.M, spec.N), dtype=torch.bfloat16, device="cuda")
    bias = wl.make_bias(spec) if spec.name in WITH_BIAS else None
    cr.convlinear4bit_forward(xd, wq, ws, g, y, ws_buf, bias=None if bias is None else to_dev_bf16(bias))
    xq, xs = cr.convrot_rotquant_act(xd, g)
    torch.cuda.synchronize()
    # the fused call leaves the activation codes and scales in its workspace: same bytes as the stand-alone call
    nb = cr.packed_bytes(spec.M, spec.K)
    assert xq.numel() == nb and torch.equal(ws_buf[:nb], xq)
    assert torch.equal(ws_buf[nb:nb + 4 * spec.M].view(torch.float32), xs)

    # ---- kernel A in full: weights and activations
    qwo, swo = oracle.rotquant(w, g)
    qwg = unpack_host(wq, spec.N, spec.K)
    fw, _ = check_codes(qwg, ws.cpu().numpy(), qwo, swo, f"{spec.name} W")
    qxo, sxo = oracle.rotquant(x, g)
    qxg = unpack_host(xq, spec.M, spec.K)
    fx, _ = check_codes(qxg, xs.cpu().numpy(), qxo, sxo, f"{spec.name} X")
    nz = np.abs(bf16_bits := wl.bf16_bits_to_f32(x)).max(axis=1) > 0
    assert (np.abs(qxg).max(axis=1)[nz] == 7).all()
    print(f"  codes identical: W {fw:.6%}  X {fx:.6%}", flush=True)
    del bf16_bits

    # ---- kernel B: integer accumulators of the whole problem, bit-exact on the GPU's own codes; bf16 output
    # of the real forward against the oracle's end-to-end value.  All rows when the oracle finishes them in
    # seconds, else a sample.
    whole = spec.M <= 4608
    rows = np.arange(spec.M) if whole else sample_rows(spec.M, seed=spec.K + spec.N)
    rt = torch.from_numpy(rows).cuda()
    acc_g = cr.convrot_w4a4_gemm_i32(xq, wq, spec.M, spec.N, spec.K)       # full-size launch
    torch.cuda.synchronize()
    acc_g = (acc_g if whole else acc_g[rt]).cpu().numpy()
    acc_o = oracle.int_gemm(qxg[rows], qwg)
    assert np.array_equal(acc_g, acc_o), f"{spec.name}: int32 GEMM differs"
    del acc_g

    if not (fw == 1.0 and fx == 1.0):
        acc_o = oracle.int_gemm(qxo[rows], qwo)
    y_o = oracle.dequant(acc_o, sxo[rows], swo, bias)
    y_g = bf16_to_host_bits(y if whole else y[rt])
    rel, cos = check_output(y_g, y_o, spec.name)
    same_rows = (qxg[rows] == qxo[rows]).all(axis=1)
    if fw == 1.0 and same_rows.any() and bias is None:
        d = bf16_ulp_diff(y_g[same_rows], y_o[same_rows])
        assert d.max() <= 1, f"{spec.name}: output {d.max()} bf16 steps off on identical codes"
    assert torch.isfinite(y.float()).all()
    print(f"  integer GEMM exact and output max rel err {rel:.3e}, cosine {cos:.7f} on "
          f"{'all' if whole else len(rows)} rows", flush=True)
