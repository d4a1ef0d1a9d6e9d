"""ctypes binding of libconvrot: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and streams, nothing
else); every step of the path runs inside the library's kernels.  There is no fallback: if the
shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconvrot.so")

STATUS_NAMES = {0: "CONVROT_OK", -1: "CONVROT_ERR_NULL", -2: "CONVROT_ERR_SHAPE", -3: "CONVROT_ERR_GROUP",
                -4: "CONVROT_ERR_ALIGN", -5: "CONVROT_ERR_WORKSPACE", -6: "CONVROT_ERR_HIP"}

# every symbol include/convrot.h declares
EXPORTS = ("convrot_status_string", "convrot_version", "convrot_packed_bytes", "convrot_workspace_bytes",
           "convrot_prepare_weight", "convrot_rotquant_act", "convrot_w4a4_gemm_dequant",
           "convlinear4bit_forward", "convrot_w4a4_gemm_i32",
           "convrot_prepare_weight8", "convrot_rotquant_act8", "convrot_w8a8_gemm_dequant",
           "convlinear8bit_forward", "convrot_w8a8_gemm_i32", "convrot_rotated_absmax",
           "convrot_workspace_bytes8", "convrot_packed_bytes8", "convrot_unpack_codes",
           "convrot_gemm_tile_rows", "convrot_init", "convlinear4bit_forward_noalloc", "convrot_build_info")
NOALLOC_WORKSPACE_BYTES = 64 << 20

_lib = None


class ConvRotError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


def load() -> ctypes.CDLL:
    """Load libconvrot.so (built by ``python -m paper_2512_03673_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -m paper_2512_03673_amd.build` (hipcc, gfx950). "
            "There is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    lib.convrot_status_string.argtypes = [i32]
    lib.convrot_status_string.restype = ctypes.c_char_p
    lib.convrot_version.argtypes = []
    lib.convrot_version.restype = i32
    lib.convrot_packed_bytes.argtypes = [i64, i64]
    lib.convrot_packed_bytes.restype = sz
    lib.convrot_workspace_bytes.argtypes = [i64, i64]
    lib.convrot_workspace_bytes.restype = sz
    lib.convrot_prepare_weight.argtypes = [vp, i64, i64, i32, vp, vp, vp]
    lib.convrot_rotquant_act.argtypes = [vp, i64, i64, i32, vp, vp, vp]
    lib.convrot_w4a4_gemm_dequant.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp, vp]
    lib.convlinear4bit_forward.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, sz, vp]
    lib.convrot_w4a4_gemm_i32.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    lib.convrot_workspace_bytes8.argtypes = [i64, i64]
    lib.convrot_workspace_bytes8.restype = sz
    lib.convrot_prepare_weight8.argtypes = lib.convrot_prepare_weight.argtypes
    lib.convrot_rotquant_act8.argtypes = lib.convrot_rotquant_act.argtypes
    lib.convrot_w8a8_gemm_dequant.argtypes = lib.convrot_w4a4_gemm_dequant.argtypes
    lib.convlinear8bit_forward.argtypes = lib.convlinear4bit_forward.argtypes
    lib.convrot_w8a8_gemm_i32.argtypes = lib.convrot_w4a4_gemm_i32.argtypes
    lib.convrot_rotated_absmax.argtypes = [vp, i64, i64, i32, i32, vp, vp]
    lib.convrot_gemm_tile_rows.argtypes = [i64, i64]
    lib.convrot_gemm_tile_rows.restype = i32
    lib.convrot_packed_bytes8.argtypes = [i64, i64]
    lib.convrot_packed_bytes8.restype = sz
    lib.convrot_unpack_codes.argtypes = [vp, i64, i64, vp, vp]
    lib.convrot_unpack_codes.restype = i32
    lib.convrot_build_info.argtypes = []
    lib.convrot_build_info.restype = ctypes.c_char_p
    lib.convrot_init.argtypes = []
    lib.convrot_init.restype = i32
    lib.convlinear4bit_forward_noalloc.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, vp]
    lib.convlinear4bit_forward_noalloc.restype = i32
    for name in EXPORTS[4:15]:
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().convrot_status_string(int(status)).decode()


def version() -> int:
    return int(load().convrot_version())


def build_info() -> str:
    return load().convrot_build_info().decode()


def init() -> None:
    """convrot_init on torch's current device: loads the device code, resolves the static workspace."""
    _check(load().convrot_init(), "convrot_init")


def gemm_tile_rows(M: int, N: int) -> int:
    return int(load().convrot_gemm_tile_rows(M, N))


def packed_bytes(rows: int, K: int) -> int:
    return int(load().convrot_packed_bytes(rows, K))


def packed_bytes8(rows: int, K: int) -> int:
    return int(load().convrot_packed_bytes8(rows, K))


def workspace_bytes(M: int, K: int) -> int:
    return int(load().convrot_workspace_bytes(M, K))


def workspace_bytes8(M: int, K: int) -> int:
    return int(load().convrot_workspace_bytes8(M, K))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check(status: int, what: str) -> None:
    if status != 0:
        raise ConvRotError(status, what)


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> None:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU")


def _bias(b: Optional[torch.Tensor], N: int) -> None:
    if b is not None:
        _dev(b, torch.bfloat16, "bias")
        if b.shape != (N,):
            raise ValueError("bias: need shape [N]")


def _codes(t: torch.Tensor, nbytes: int, name: str) -> None:
    """A code matrix is an opaque uint8 buffer in the library's panel layout."""
    _dev(t, torch.uint8, name)
    if t.numel() < nbytes:
        raise ValueError(f"{name}: need {nbytes} bytes (convrot_packed_bytes), got {t.numel()}")


def _new_codes(nbytes: int, device) -> torch.Tensor:
    return torch.empty((nbytes,), dtype=torch.uint8, device=device)


def convrot_prepare_weight(W: torch.Tensor, group: int, Wq: Optional[torch.Tensor] = None,
                           w_scale: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """W bf16 [N, K] -> (Wq uint8 [packed_bytes(N, K)], w_scale f32 [N])."""
    _dev(W, torch.bfloat16, "W")
    N, K = W.shape
    Wq = _new_codes(packed_bytes(N, K), W.device) if Wq is None else Wq
    _codes(Wq, packed_bytes(N, K), "Wq")
    w_scale = torch.empty((N,), dtype=torch.float32, device=W.device) if w_scale is None else w_scale
    _check(load().convrot_prepare_weight(_ptr(W), N, K, group, _ptr(Wq), _ptr(w_scale), _stream(stream)),
           "convrot_prepare_weight")
    return Wq, w_scale


def convrot_rotquant_act(X: torch.Tensor, group: int, Xq: Optional[torch.Tensor] = None,
                         x_scale: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """X bf16 [M, K] -> (Xq uint8 [packed_bytes(M, K)], x_scale f32 [M])."""
    _dev(X, torch.bfloat16, "X")
    M, K = X.shape
    Xq = _new_codes(packed_bytes(M, K), X.device) if Xq is None else Xq
    _codes(Xq, packed_bytes(M, K), "Xq")
    x_scale = torch.empty((M,), dtype=torch.float32, device=X.device) if x_scale is None else x_scale
    _check(load().convrot_rotquant_act(_ptr(X), M, K, group, _ptr(Xq), _ptr(x_scale), _stream(stream)),
           "convrot_rotquant_act")
    return Xq, x_scale


def convrot_unpack_codes(Xq: torch.Tensor, rows: int, K: int, codes: Optional[torch.Tensor] = None,
                         stream=None) -> torch.Tensor:
    """4-bit code matrix -> int8 codes [rows, K] (gate / debug export)."""
    _codes(Xq, packed_bytes(rows, K), "Xq")
    codes = torch.empty((rows, K), dtype=torch.int8, device=Xq.device) if codes is None else codes
    _check(load().convrot_unpack_codes(_ptr(Xq), rows, K, _ptr(codes), _stream(stream)), "convrot_unpack_codes")
    return codes


def convrot_w4a4_gemm_dequant(Xq: torch.Tensor, x_scale: torch.Tensor, Wq: torch.Tensor, w_scale: torch.Tensor,
                              K: int, Y: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None,
                              stream=None) -> torch.Tensor:
    """Code matrices + scales f32 [M], [N] (+ bias bf16 [N]) -> Y bf16 [M, N]."""
    _dev(x_scale, torch.float32, "x_scale"); _dev(w_scale, torch.float32, "w_scale")
    M, N = x_scale.shape[0], w_scale.shape[0]
    _codes(Xq, packed_bytes(M, K), "Xq"); _codes(Wq, packed_bytes(N, K), "Wq")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=Xq.device) if Y is None else Y
    _bias(bias, N)
    _check(load().convrot_w4a4_gemm_dequant(_ptr(Xq), _ptr(x_scale), _ptr(Wq), _ptr(w_scale), _ptr(bias), M, N,
                                            K, _ptr(Y), _stream(stream)), "convrot_w4a4_gemm_dequant")
    return Y


def convrot_w4a4_gemm_i32(Xq: torch.Tensor, Wq: torch.Tensor, M: int, N: int, K: int,
                          acc: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Code matrices of [M, K] and [N, K] -> raw int32 accumulators [M, N] (gate / debug export)."""
    _codes(Xq, packed_bytes(M, K), "Xq"); _codes(Wq, packed_bytes(N, K), "Wq")
    acc = torch.empty((M, N), dtype=torch.int32, device=Xq.device) if acc is None else acc
    _check(load().convrot_w4a4_gemm_i32(_ptr(Xq), _ptr(Wq), M, N, K, _ptr(acc), _stream(stream)),
           "convrot_w4a4_gemm_i32")
    return acc


def convlinear4bit_forward(X: torch.Tensor, Wq: torch.Tensor, w_scale: torch.Tensor, group: int,
                           Y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           bias: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """X bf16 [M, K], prepared weight -> Y bf16 [M, N]; `workspace` is a uint8 tensor of workspace_bytes(M, K)."""
    _dev(X, torch.bfloat16, "X"); _dev(w_scale, torch.float32, "w_scale")
    M, K = X.shape
    N = w_scale.shape[0]
    _codes(Wq, packed_bytes(N, K), "Wq")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if Y is None else Y
    if workspace is None:
        workspace = torch.empty((max(workspace_bytes(M, K), 256),), dtype=torch.uint8, device=X.device)
    _bias(bias, N)
    _check(load().convlinear4bit_forward(_ptr(X), _ptr(Wq), _ptr(w_scale), _ptr(bias), M, N, K, group, _ptr(Y),
                                         _ptr(workspace), workspace.numel(), _stream(stream)),
           "convlinear4bit_forward")
    return Y


def convlinear4bit_forward_noalloc(X: torch.Tensor, Wq: torch.Tensor, w_scale: torch.Tensor, group: int,
                                   Y: torch.Tensor, bias: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """As convlinear4bit_forward, the activation codes in the library's static device array; `Y` is the caller's."""
    _dev(X, torch.bfloat16, "X"); _dev(w_scale, torch.float32, "w_scale"); _dev(Y, torch.bfloat16, "Y")
    M, K = X.shape
    N = w_scale.shape[0]
    if Y.shape != (M, N):
        raise ValueError("Y: need shape [M, N]")
    _codes(Wq, packed_bytes(N, K), "Wq")
    _bias(bias, N)
    _check(load().convlinear4bit_forward_noalloc(_ptr(X), _ptr(Wq), _ptr(w_scale), _ptr(bias), M, N, K, group,
                                                 _ptr(Y), _stream(stream)), "convlinear4bit_forward_noalloc")
    return Y


ROT_NONE, ROT_REGULAR, ROT_SYLVESTER = 0, 1, 2


def convrot_rotated_absmax(X: torch.Tensor, group: int, kind: int, out: Optional[torch.Tensor] = None,
                           stream=None) -> torch.Tensor:
    """Per-row max |R(X)| for kind ROT_NONE / ROT_REGULAR / ROT_SYLVESTER (diagnostic) -> f32 [M]."""
    _dev(X, torch.bfloat16, "X")
    M, K = X.shape
    out = torch.empty((M,), dtype=torch.float32, device=X.device) if out is None else out
    _check(load().convrot_rotated_absmax(_ptr(X), M, K, group, kind, _ptr(out), _stream(stream)),
           "convrot_rotated_absmax")
    return out


# ---------------------------------------------------------------------------- W8A8 variant
def _rotquant8(fn_name: str, X: torch.Tensor, group: int, Xq, x_scale, stream):
    _dev(X, torch.bfloat16, "input")
    rows, K = X.shape
    Xq = _new_codes(packed_bytes8(rows, K), X.device) if Xq is None else Xq
    _codes(Xq, packed_bytes8(rows, K), "codes")
    x_scale = torch.empty((rows,), dtype=torch.float32, device=X.device) if x_scale is None else x_scale
    _check(getattr(load(), fn_name)(_ptr(X), rows, K, group, _ptr(Xq), _ptr(x_scale), _stream(stream)), fn_name)
    return Xq, x_scale


def convrot_prepare_weight8(W: torch.Tensor, group: int, Wq: Optional[torch.Tensor] = None,
                            w_scale: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """W bf16 [N, K] -> (Wq uint8 [packed_bytes8(N, K)], w_scale f32 [N])."""
    return _rotquant8("convrot_prepare_weight8", W, group, Wq, w_scale, stream)


def convrot_rotquant_act8(X: torch.Tensor, group: int, Xq: Optional[torch.Tensor] = None,
                          x_scale: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """X bf16 [M, K] -> (Xq uint8 [packed_bytes8(M, K)], x_scale f32 [M])."""
    return _rotquant8("convrot_rotquant_act8", X, group, Xq, x_scale, stream)


def convrot_w8a8_gemm_dequant(Xq: torch.Tensor, x_scale: torch.Tensor, Wq: torch.Tensor, w_scale: torch.Tensor,
                              K: int, Y: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None,
                              stream=None) -> torch.Tensor:
    """8-bit code matrices + scales f32 [M], [N] (+ bias bf16 [N]) -> Y bf16 [M, N]."""
    _dev(x_scale, torch.float32, "x_scale"); _dev(w_scale, torch.float32, "w_scale")
    M, N = x_scale.shape[0], w_scale.shape[0]
    _codes(Xq, packed_bytes8(M, K), "Xq"); _codes(Wq, packed_bytes8(N, K), "Wq")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=Xq.device) if Y is None else Y
    _bias(bias, N)
    _check(load().convrot_w8a8_gemm_dequant(_ptr(Xq), _ptr(x_scale), _ptr(Wq), _ptr(w_scale), _ptr(bias), M, N, K,
                                            _ptr(Y), _stream(stream)), "convrot_w8a8_gemm_dequant")
    return Y


def convrot_w8a8_gemm_i32(Xq: torch.Tensor, Wq: torch.Tensor, M: int, N: int, K: int,
                          acc: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """8-bit code matrices of [M, K] and [N, K] -> raw int32 accumulators [M, N] (gate / debug export)."""
    _codes(Xq, packed_bytes8(M, K), "Xq"); _codes(Wq, packed_bytes8(N, K), "Wq")
    acc = torch.empty((M, N), dtype=torch.int32, device=Xq.device) if acc is None else acc
    _check(load().convrot_w8a8_gemm_i32(_ptr(Xq), _ptr(Wq), M, N, K, _ptr(acc), _stream(stream)),
           "convrot_w8a8_gemm_i32")
    return acc


def convlinear8bit_forward(X: torch.Tensor, Wq: torch.Tensor, w_scale: torch.Tensor, group: int,
                           Y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           bias: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """X bf16 [M, K], prepared 8-bit weight -> Y bf16 [M, N]; `workspace`: uint8 tensor of workspace_bytes8(M, K)."""
    _dev(X, torch.bfloat16, "X"); _dev(w_scale, torch.float32, "w_scale")
    M, K = X.shape
    N = w_scale.shape[0]
    _codes(Wq, packed_bytes8(N, K), "Wq")
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device) if Y is None else Y
    if workspace is None:
        workspace = torch.empty((max(workspace_bytes8(M, K), 256),), dtype=torch.uint8, device=X.device)
    _bias(bias, N)
    _check(load().convlinear8bit_forward(_ptr(X), _ptr(Wq), _ptr(w_scale), _ptr(bias), M, N, K, group, _ptr(Y),
                                         _ptr(workspace), workspace.numel(), _stream(stream)),
           "convlinear8bit_forward")
    return Y
