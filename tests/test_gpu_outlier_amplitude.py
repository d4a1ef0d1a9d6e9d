"""The outlier-amplitude diagnostic max |X H| (Sec. 4.2, Table 5-1, Fig. 3-2) on the GPU against the oracle's
rotation with an explicit matrix, and the paper's qualitative claim on synthetic one-signed activations."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import to_dev_bf16
from paper_2512_03673_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cr():
    from paper_2512_03673_amd import binding
    binding.load()
    return binding


def sylvester(g: int) -> np.ndarray:
    H = np.array([[1]], dtype=np.int8)
    while H.shape[0] < g:
        H = np.kron(np.array([[1, 1], [1, -1]], dtype=np.int8), H)
    return H


def oracle_amplitude(x_bits, g, kind):
    if kind == 0:
        return np.abs(wl.bf16_bits_to_f32(x_bits).astype(np.float64)).max(axis=1)
    H = oracle.hadamard(g) if kind == 1 else sylvester(g)
    return np.abs(oracle.rotate(x_bits, g, H)).max(axis=1)


@pytest.mark.parametrize("g", (4, 16, 64, 256, 1024))
@pytest.mark.parametrize("kind", (0, 1, 2))
@pytest.mark.parametrize("M,K", [(37, 1024), (5, 3072), (9, 15360), (3, 2048)])
def test_rotated_absmax_matches_oracle(cr, g, kind, M, K):
    if K % g:
        pytest.skip("K not a multiple of g")
    spec = wl.LayerSpec(f"amp_{M}_{K}", M=M, K=K, N=8, group=g, x_kind="halfnormal", x_col_count=max(1, K // 100),
                        x_row_count=1, seed=21)
    x = wl.make_activation(spec)
    a = cr.convrot_rotated_absmax(to_dev_bf16(x), g, kind)
    torch.cuda.synchronize()
    want = oracle_amplitude(x, g, kind)
    assert np.allclose(a.cpu().numpy().astype(np.float64), want, rtol=2e-6, atol=0)


def test_regular_amplitude_is_seven_times_the_scale(cr):
    spec = wl.LayerSpec("amp_scale", M=64, K=3072, N=8, group=16, seed=22)
    x = to_dev_bf16(wl.make_activation(spec))
    a = cr.convrot_rotated_absmax(x, 16, cr.ROT_REGULAR).cpu().numpy()
    _, s = cr.convrot_rotquant_act(x, 16)
    assert np.array_equal((a / np.float32(7.0)).astype(np.float32), s.cpu().numpy())


def test_sylvester_amplifies_one_signed_rows_regular_does_not(cr):
    # the GELU-like down-projection input of configuration 3: non-negative activations with row outliers.
    # A constant row c maps to c sqrt(g) in the Sylvester matrix's first output and to c in the regular one's.
    spec = wl.CONFIGS["cfg3_mlp"][1]
    x = to_dev_bf16(wl.make_activation(spec, rows=512))
    amp = {g: {k: float(cr.convrot_rotated_absmax(x, g, k).max()) for k in (0, 1, 2)} for g in (16, 64, 256, 1024)}
    torch.cuda.synchronize()
    for g, a in amp.items():
        print(f"g={g}: none {a[0]:.1f}  regular {a[1]:.1f}  sylvester {a[2]:.1f}", flush=True)
        assert a[1] < a[2]                       # Sylvester is worse than regular at every group size
    # a larger group spreads a channel outlier thinner (1 / sqrt(g)): the regular matrix's amplitude keeps falling,
    # while the Sylvester matrix's turns around as the one-signed outlier rows add up (sqrt(g)) - the shape of
    # the paper's Table 5-1; the ratio between the two grows with g
    assert amp[16][1] > amp[64][1] > amp[256][1] > amp[1024][1]
    assert amp[1024][2] > amp[256][2] > amp[64][2]
    ratio = [amp[g][2] / amp[g][1] for g in (16, 64, 256, 1024)]
    assert ratio == sorted(ratio) and ratio[-1] > 1.8
    assert all(a[1] < a[0] for a in amp.values())          # and the rotation always beats no rotation here
    c = torch.full((2, 1024), 3.0, dtype=torch.bfloat16, device="cuda")
    assert cr.convrot_rotated_absmax(c, 1024, cr.ROT_SYLVESTER)[0].item() == 3.0 * 32
    assert cr.convrot_rotated_absmax(c, 1024, cr.ROT_REGULAR)[0].item() == 3.0
