"""GPU: the library launches on the stream it is given, calls on different streams do not disturb each other,
and a forward can be captured into a HIP graph and replayed (it allocates nothing and records no memset).

The expected outputs are the library's own results on the default stream, which the parity tests hold
against the oracle; one case here is checked against the oracle directly as well.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import bf16_to_host_bits, check_output, to_dev_bf16
from paper_2512_03673_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cr():
    from paper_2512_03673_amd import binding
    binding.load()
    return binding


def layer(M, K, N, g, seed):
    spec = wl.LayerSpec(f"stream_{seed}", M=M, K=K, N=N, group=g, seed=seed)
    x, w = wl.make_layer(spec)
    return spec, x, w


def test_forward_runs_on_the_given_stream(cr):
    # X is produced on a side stream by a long chain of kernels; the forward is queued behind it on the same
    # stream.  Launched anywhere else it would read X before the chain has written it (torch's side streams
    # do not synchronise with the default stream).
    spec, x, w = layer(300, 1024, 520, 16, 11)
    X = to_dev_bf16(x)
    wq, ws = cr.convrot_prepare_weight(to_dev_bf16(w), 16)
    y_ref = cr.convlinear4bit_forward(X, wq, ws, 16)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    Xs = torch.zeros_like(X)
    big = torch.ones((8192, 8192), device="cuda")
    Y = torch.zeros_like(y_ref)
    wsb = torch.empty((cr.workspace_bytes(spec.M, spec.K),), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(20):
            big = big * 1.0001 + 0.5          # milliseconds of work ahead of the copy
        Xs.copy_(X)
        cr.convlinear4bit_forward(Xs, wq, ws, 16, Y, wsb, stream=side)
    side.synchronize()
    assert torch.equal(Y, y_ref)
    (qx, sx), (qw, sw) = oracle.rotquant(x, 16), oracle.rotquant(w, 16)
    yo = oracle.dequant(oracle.int_gemm(qx, qw), sx, sw)
    check_output(bf16_to_host_bits(Y), yo, "forward on a side stream")


def test_calls_on_two_streams_do_not_disturb_each_other(cr):
    # two layers of different shape (one per block tile shape of the GEMM), each with its own buffers, queued
    # alternately on two streams
    cases = []
    for M, K, N, g, seed in ((3072, 256, 3072, 16, 21), (700, 2048, 900, 64, 22)):
        spec, x, w = layer(M, K, N, g, seed)
        X = to_dev_bf16(x)
        wq, ws = cr.convrot_prepare_weight(to_dev_bf16(w), g)
        y_ref = cr.convlinear4bit_forward(X, wq, ws, g)
        Y = torch.empty_like(y_ref)
        wsb = torch.empty((cr.workspace_bytes(M, K),), dtype=torch.uint8, device="cuda")
        cases.append((X, wq, ws, g, Y, wsb, y_ref, torch.cuda.Stream()))
    assert cr.gemm_tile_rows(3072, 3072) == 192 and cr.gemm_tile_rows(700, 900) == 256
    torch.cuda.synchronize()
    for rep in range(10):
        for X, wq, ws, g, Y, wsb, y_ref, s in cases:
            with torch.cuda.stream(s):
                if rep == 9:
                    Y.zero_()
                cr.convlinear4bit_forward(X, wq, ws, g, Y, wsb, stream=s)
    torch.cuda.synchronize()
    for X, wq, ws, g, Y, wsb, y_ref, s in cases:
        assert torch.equal(Y, y_ref)


@pytest.mark.parametrize("bits", (4, 8))
def test_forward_in_a_hip_graph(cr, bits):
    spec, x, w = layer(520, 1024, 300, 16, 31 + bits)
    prep, fwd, wsbytes = ((cr.convrot_prepare_weight, cr.convlinear4bit_forward, cr.workspace_bytes) if bits == 4 else
                          (cr.convrot_prepare_weight8, cr.convlinear8bit_forward, cr.workspace_bytes8))
    X = to_dev_bf16(x)
    wq, ws = prep(to_dev_bf16(w), 16)
    bias = to_dev_bf16(wl.make_bias(spec))
    Y = torch.zeros((spec.M, spec.N), dtype=torch.bfloat16, device="cuda")
    wsb = torch.empty((wsbytes(spec.M, spec.K),), dtype=torch.uint8, device="cuda")
    y_eager = fwd(X, wq, ws, 16, bias=bias).clone()     # also the first launch: sets the kernels' LDS limits
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fwd(X, wq, ws, 16, Y, wsb, bias=bias)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for rep in range(4):
        # new input in the captured buffer, eager work and a synchronisation between the replays
        x2 = wl.f32_to_bf16_bits((rng.standard_normal((spec.M, spec.K)) * (rep + 1)).astype(np.float32))
        X.copy_(to_dev_bf16(x2))
        y_eager = fwd(X, wq, ws, 16, bias=bias).clone()
        Y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, y_eager), f"replay {rep}"
