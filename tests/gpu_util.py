"""Helpers shared by the GPU parity tests: host <-> device marshalling and the parity gates."""
import numpy as np
import torch


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 tensor on the GPU (no value conversion)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_host_bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def from_panels(buf: np.ndarray, rows: int, row_bytes: int) -> np.ndarray:
    """The library's code-matrix layout (1 KB panels of 16 rows x 64 bytes, K-panels of the same rows
    adjacent) -> row-major uint8 [rows, row_bytes].  Checks that the K padding holds zero codes."""
    rp, kp = -(-rows // 16), -(-row_bytes // 64)
    buf = np.ascontiguousarray(buf).view(np.uint8).ravel()
    assert buf.size >= rp * kp * 1024, "code matrix shorter than its panel layout"
    a = buf[:rp * kp * 1024].reshape(rp, kp, 16, 64).transpose(0, 2, 1, 3).reshape(rp * 16, kp * 64)
    assert not a[:rows, row_bytes:].any(), "K padding of a code matrix must be zero codes"
    return np.ascontiguousarray(a[:rows, :row_bytes])


def to_panels(mat: np.ndarray, junk: int = 0x5A) -> np.ndarray:
    """Row-major byte matrix -> panel layout.  The K padding is zero, as the library requires; the padding
    rows of the last row panel are filled with `junk`, which the library must never look at."""
    mat = np.ascontiguousarray(mat).view(np.uint8)
    rows, row_bytes = mat.shape
    rp, kp = -(-rows // 16), -(-row_bytes // 64)
    a = np.full((rp * 16, kp * 64), junk, dtype=np.uint8)
    a[:rows] = 0
    a[:rows, :row_bytes] = mat
    return np.ascontiguousarray(a.reshape(rp, 16, kp, 64).transpose(0, 2, 1, 3)).ravel()


def unpack_nibbles(packed: np.ndarray) -> np.ndarray:
    """Row-major packed 4-bit codes [rows, K/2] -> int8 codes [rows, K] (numpy, test side)."""
    lo = (packed & 0xF).astype(np.int8)
    hi = (packed >> 4).astype(np.int8)
    lo = np.where(lo >= 8, lo - 16, lo).astype(np.int8)
    hi = np.where(hi >= 8, hi - 16, hi).astype(np.int8)
    out = np.empty((packed.shape[0], packed.shape[1] * 2), dtype=np.int8)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out


def unpack_host(buf, rows: int, K: int) -> np.ndarray:
    """4-bit code matrix as the library stores it (tensor or array) -> int8 codes [rows, K]."""
    if isinstance(buf, torch.Tensor):
        buf = buf.cpu().numpy()
    return unpack_nibbles(from_panels(buf, rows, K // 2))


def unpack_host8(buf, rows: int, K: int) -> np.ndarray:
    """8-bit code matrix as the library stores it -> int8 codes [rows, K]."""
    if isinstance(buf, torch.Tensor):
        buf = buf.cpu().numpy()
    return from_panels(buf, rows, K).view(np.int8)


def codes4_to_dev(codes: np.ndarray) -> torch.Tensor:
    """int8 codes [rows, K] in [-7, 7] -> 4-bit code matrix on the GPU, in the library's layout."""
    c = codes.astype(np.uint8) & 0xF
    packed = (c[:, 0::2] | (c[:, 1::2] << 4)).astype(np.uint8)
    return torch.from_numpy(to_panels(packed)).cuda()


def codes8_to_dev(codes: np.ndarray) -> torch.Tensor:
    """int8 codes [rows, K] -> 8-bit code matrix on the GPU, in the library's layout."""
    return torch.from_numpy(to_panels(codes.astype(np.int8).view(np.uint8))).cuda()


def ulp_diff_f32(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    ia = a.view(np.int32).astype(np.int64)
    ib = b.view(np.int32).astype(np.int64)
    return np.abs(ia - ib)


def check_codes(codes_gpu: np.ndarray, scale_gpu: np.ndarray, codes_ref: np.ndarray, scale_ref: np.ndarray,
                what: str = ""):
    """Gate: codes identical on >= 99.99 % of elements, never more than 1 LSB apart; scales within 2 fp32 ulp."""
    assert codes_gpu.shape == codes_ref.shape, what
    d = np.abs(codes_gpu.astype(np.int16) - codes_ref.astype(np.int16))
    frac = float((d == 0).mean()) if d.size else 1.0
    assert d.size == 0 or d.max() <= 1, f"{what}: code off by {d.max()} LSB"
    assert frac >= 0.9999, f"{what}: only {frac:.6%} of codes identical"
    assert np.abs(codes_gpu).max(initial=0) <= 7, what
    u = ulp_diff_f32(scale_gpu, scale_ref)
    assert u.size == 0 or u.max() <= 2, f"{what}: scale off by {u.max()} ulp"
    return frac, float((u == 0).mean()) if u.size else 1.0


def check_output(y_gpu_bits: np.ndarray, y_ref_bits: np.ndarray, what: str = ""):
    """Gate: max |Y - Yo| / max |Yo| <= 1e-2 and cosine similarity >= 0.9999."""
    y, r = bits_to_f64(y_gpu_bits).ravel(), bits_to_f64(y_ref_bits).ravel()
    assert np.isfinite(y).all(), what
    denom = np.abs(r).max()
    rel = float(np.abs(y - r).max() / denom) if denom > 0 else float(np.abs(y).max())
    nr, ny = np.linalg.norm(r), np.linalg.norm(y)
    cos = float(y @ r / (nr * ny)) if nr > 0 and ny > 0 else 1.0
    assert rel <= 1e-2, f"{what}: max rel err {rel}"
    assert cos >= 0.9999, f"{what}: cosine {cos}"
    return rel, cos


def bf16_ulp_diff(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in bf16 steps between two bf16 bit arrays (sign-magnitude aware)."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))
