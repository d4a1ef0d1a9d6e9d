"""GPU: the library launches on the stream it is given, calls on different streams do not disturb each other,
and a forward can be captured into a HIP graph and replayed (it allocates nothing and records no memset).

The expected outputs are the library's own results on the default stream, which the parity tests hold
against the oracle; one case here is checked against the oracle directly as well.
"""
import os
import subprocess
import sys

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


_FIRST_CALL_CAPTURED = r"""
import sys
import torch
sys.path.insert(0, sys.argv[1])
from paper_2512_03673_amd import binding as cr
bits = int(sys.argv[2])
fwd, packed, wsbytes = ((cr.convlinear4bit_forward, cr.packed_bytes, cr.workspace_bytes) if bits == 4 else
                        (cr.convlinear8bit_forward, cr.packed_bytes8, cr.workspace_bytes8))
M, K, N, g = 520, 1024, 3000, 16
torch.manual_seed(3)
X = torch.randn((M, K), device="cuda").to(torch.bfloat16)
# any bytes are a valid code matrix (every six-bit pattern is a finite E2M3 number, every byte an int8 code), so the
# weight needs no library call; the K padding must hold zero codes, and K = 1024 has none
wq = torch.randint(0, 256, (packed(N, K),), dtype=torch.uint8, device="cuda")
ws = torch.rand((N,), device="cuda") * 1e-3 + 1e-4
bias = torch.randn((N,), device="cuda").to(torch.bfloat16)
Y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
wsb = torch.empty((wsbytes(M, K),), dtype=torch.uint8, device="cuda")
torch.cuda.synchronize()
graph = torch.cuda.CUDAGraph()
with torch.cuda.graph(graph):                       # the first call into the library in this process
    fwd(X, wq, ws, g, Y, wsb, bias=bias)
for rep in range(3):
    X.copy_(torch.randn((M, K), device="cuda").to(torch.bfloat16) * (rep + 1))
    Y.zero_()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    y_eager = fwd(X, wq, ws, g, bias=bias)
    torch.cuda.synchronize()
    assert torch.isfinite(Y.float()).all() and Y.float().abs().max() > 0
    assert torch.equal(Y, y_eager), f"replay {rep}"
print("first call captured: ok")
"""


@pytest.mark.parametrize("bits", (4, 8))
def test_first_library_call_of_a_process_under_capture(bits):
    # The library keeps no set-up for a first eager call to do: a process whose very first call into it is made
    # under stream capture gets a working graph.  Run in a child process, which has not touched the library.
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", _FIRST_CALL_CAPTURED, root, str(bits)], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode == 0 and "first call captured: ok" in r.stdout, r.stdout + r.stderr
