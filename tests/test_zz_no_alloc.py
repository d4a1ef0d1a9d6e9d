"""GPU: convlinear4bit_forward_noalloc (activation codes in the library's static device array) against
convlinear4bit_forward with a caller's workspace: bit-identical output, on consecutive calls that share the
array, the later ones with smaller inputs; limits and errors; and inside a HIP graph."""
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


def make(cr, M, K, N, g, seed, with_bias):
    spec = wl.LayerSpec(f"noalloc_{seed}", M=M, K=K, N=N, group=g, seed=seed)
    x, w = wl.make_layer(spec)
    wq, ws = cr.convrot_prepare_weight(to_dev_bf16(w), g)
    bias = wl.make_bias(spec) if with_bias else None
    return spec, x, w, to_dev_bf16(x), wq, ws, bias


def test_noalloc_matches_forward_on_consecutive_calls(cr):
    # large, then smaller, then a ragged small one whose last 32-row block keeps rows of the earlier calls, then large
    # again: every call finds the previous call's codes and scales in the array
    shapes = [(4608, 3072, 3072, 16, True), (1000, 2048, 520, 64, False), (37, 96, 200, 16, True),
              (300, 1024, 520, 256, False), (4608, 3072, 3072, 16, True)]
    for i, (M, K, N, g, with_bias) in enumerate(shapes):
        print(f"case {i}: M={M} K={K} N={N} g={g}", flush=True)
        spec, x, w, X, wq, ws, bias = make(cr, M, K, N, g, 40 + i, with_bias)
        b = None if bias is None else to_dev_bf16(bias)
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        cr.convlinear4bit_forward_noalloc(X, wq, ws, g, Y, bias=b)
        y_ref = cr.convlinear4bit_forward(X, wq, ws, g, bias=b)
        torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), y_ref.view(torch.int16)), f"case {i}"
        if M <= 1000:
            check_output(bf16_to_host_bits(Y), oracle.convlinear4bit(x, w, g, bias=bias), f"noalloc case {i}")


def test_noalloc_limit_and_errors(cr):
    lib = cr.load()
    limit = cr.NOALLOC_WORKSPACE_BYTES
    assert cr.workspace_bytes(4608, 15360) <= limit < cr.workspace_bytes(16896, 12288)
    dev = torch.device("cuda")
    K = 12288
    M = 16896                                   # needs 156 MB of workspace: beyond the static array
    X = torch.zeros((M, K), dtype=torch.bfloat16, device=dev)
    wq = torch.zeros((cr.packed_bytes(8, K),), dtype=torch.uint8, device=dev)
    ws = torch.ones((8,), dtype=torch.float32, device=dev)
    Y = torch.full((M, 8), 3.0, dtype=torch.bfloat16, device=dev)
    with pytest.raises(cr.ConvRotError) as e:
        cr.convlinear4bit_forward_noalloc(X, wq, ws, 16, Y)
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert (Y == 3.0).all()                     # nothing was launched
    # the same argument checks as the call with a workspace
    assert lib.convlinear4bit_forward_noalloc(None, wq.data_ptr(), ws.data_ptr(), None, 4, 8, K, 16, Y.data_ptr(), None) == -1
    assert lib.convlinear4bit_forward_noalloc(X.data_ptr(), wq.data_ptr(), ws.data_ptr(), None, 4, 8, K, 8, Y.data_ptr(), None) == -3
    assert lib.convlinear4bit_forward_noalloc(X.data_ptr() + 2, wq.data_ptr(), ws.data_ptr(), None, 4, 8, K, 16, Y.data_ptr(), None) == -4
    assert lib.convlinear4bit_forward_noalloc(X.data_ptr(), wq.data_ptr(), ws.data_ptr(), None, 4, 8, K + 16, 16, Y.data_ptr(), None) == -2
    # empty problems are no-ops
    assert lib.convlinear4bit_forward_noalloc(None, wq.data_ptr(), ws.data_ptr(), None, 0, 8, K, 16, None, None) == 0
    cr.init()
    cr.init()                                   # idempotent


def test_noalloc_in_a_hip_graph(cr):
    spec, x, w, X, wq, ws, bias = make(cr, 520, 1024, 300, 16, 77, True)
    b = to_dev_bf16(bias)
    Y = torch.zeros((spec.M, spec.N), dtype=torch.bfloat16, device="cuda")
    cr.init()                                   # the array's address is looked up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cr.convlinear4bit_forward_noalloc(X, wq, ws, 16, Y, bias=b)
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    for rep in range(4):
        x2 = wl.f32_to_bf16_bits((rng.standard_normal((spec.M, spec.K)) * (rep + 1)).astype(np.float32))
        X.copy_(to_dev_bf16(x2))
        # an eager call of another shape in between leaves its own codes in the shared array
        other = make(cr, 100 + 50 * rep, 2048, 64, 16, 90 + rep, False)
        cr.convlinear4bit_forward_noalloc(other[3], other[4], other[5], 16,
                                          torch.empty((other[0].M, 64), dtype=torch.bfloat16, device="cuda"))
        y_eager = cr.convlinear4bit_forward(X, wq, ws, 16, bias=b).clone()
        Y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, y_eager), f"replay {rep}"


def test_init_from_many_host_threads(cr):
    # convrot_init is idempotent and may be raced: every thread gets CONVROT_OK and the array's address is taken once;
    # the entry point works afterwards
    import threading
    results = []

    def worker():
        try:
            cr.init()
            results.append(0)
        except Exception as e:          # noqa: BLE001 - reported through the assertion below
            results.append(e)

    threads = [threading.Thread(target=worker) for _ in range(16)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert results == [0] * 16, results
    spec, x, w, X, wq, ws, bias = make(cr, 70, 256, 200, 16, 61, False)
    Y = cr.convlinear4bit_forward_noalloc(X, wq, ws, 16, torch.empty((70, 200), dtype=torch.bfloat16, device="cuda"))
    y_ref = cr.convlinear4bit_forward(X, wq, ws, 16)
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.int16), y_ref.view(torch.int16))
