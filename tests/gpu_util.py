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


# ---- 4-bit codes as the library stores them: FP6 (E2M3) numbers in 3 KB blocks of 32 rows x 128 codes.
# Written from the layout's description (include/convrot.h), independently of the library's own code:
#   unit   16 codes = 96 bits, code e of the unit at bit 6 * (2 * (e % 8) + e // 8)
#   chunk  an even unit followed by the odd unit after it = 24 bytes: A part = bytes 0-15, B part = bytes 16-23
#   block  32 rows x 4 chunks: A part of chunk c of row r at r*64 + ((c ^ swz_a(r)) * 16),
#          B part at 2048 + r*32 + ((c ^ swz_b(r)) * 8); swz_a(r) = ((r>>1) ^ (r>>3)) & 3, swz_b(r) = (r>>3) & 3
#   matrix block (R, S) of rows 32R.. and codes 128S.. at (R * stages + S) * 3072
_E2M3_MAG = np.array([0, 0b01000, 0b10000, 0b10100, 0b11000, 0b11010, 0b11100, 0b11110], dtype=np.uint8)   # |q| -> e2m3 bits
_E2M3_VAL = {int(bits): mag for mag, bits in enumerate(_E2M3_MAG)}


def _unit_field_order() -> np.ndarray:
    """field index (position in the 96-bit string, in units of 6 bits) of code e of a unit"""
    e = np.arange(16)
    return 2 * (e % 8) + e // 8


def _swz_a(r):
    return ((r >> 1) ^ (r >> 3)) & 3


def _swz_b(r):
    return (r >> 3) & 3


def _chunk_byte_index(rows_pad: int, stages: int):
    """For every (row, stage, chunk): start offsets of its A part and B part in the matrix buffer."""
    r = np.arange(rows_pad)[:, None, None]
    st = np.arange(stages)[None, :, None]
    c = np.arange(4)[None, None, :]
    base = ((r // 32) * stages + st) * 3072
    r32 = r % 32
    a = base + r32 * 64 + ((c ^ _swz_a(r32)) * 16)
    b = base + 2048 + r32 * 32 + ((c ^ _swz_b(r32)) * 8)
    return a, b


def encode_e2m3(codes: np.ndarray, junk: int = 0x5A) -> np.ndarray:
    """int8 codes [rows, K] in [-7, 7] -> the library's 4-bit code matrix (uint8 buffer).  The K padding of the
    last stage is zero codes, as the library requires; the rows past `rows` of the last block are `junk`."""
    rows, K = codes.shape
    stages, rows_pad = -(-K // 128), -(-rows // 32) * 32
    c = np.zeros((rows, stages * 128), dtype=np.int8)
    c[:, :K] = codes
    fp6 = (_E2M3_MAG[np.abs(c)] | np.where(c < 0, 32, 0)).astype(np.uint8)            # [rows, Kpad] 6-bit values
    units = fp6.reshape(rows, stages * 8, 16)
    bits = np.zeros((rows, stages * 8, 96), dtype=np.uint8)                              # bit strings, LSB first
    order = _unit_field_order()
    for e in range(16):
        for k in range(6):
            bits[:, :, 6 * order[e] + k] = (units[:, :, e] >> k) & 1
    unit_bytes = np.packbits(bits, axis=2, bitorder="little")                           # [rows, units, 12]
    chunk = unit_bytes.reshape(rows, stages, 4, 24)
    buf = np.full(rows_pad // 32 * stages * 3072, junk, dtype=np.uint8)
    a, b = _chunk_byte_index(rows_pad, stages)
    ai = (a[:rows, :, :, None] + np.arange(16)).ravel()
    bi = (b[:rows, :, :, None] + np.arange(8)).ravel()
    buf[ai] = chunk[:, :, :, :16].ravel()
    buf[bi] = chunk[:, :, :, 16:].ravel()
    return buf


def decode_e2m3(buf: np.ndarray, rows: int, K: int) -> np.ndarray:
    """The library's 4-bit code matrix -> int8 codes [rows, K].  Checks that every 6-bit field is one of the 15
    codes (a negative zero is accepted as 0) and that the K padding holds zero codes."""
    stages, rows_pad = -(-K // 128), -(-rows // 32) * 32
    buf = np.ascontiguousarray(buf).view(np.uint8).ravel()
    assert buf.size >= rows_pad // 32 * stages * 3072, "code matrix shorter than its layout"
    a, b = _chunk_byte_index(rows_pad, stages)
    ai = a[:rows, :, :, None] + np.arange(16)
    bi = b[:rows, :, :, None] + np.arange(8)
    chunk = np.concatenate([buf[ai], buf[bi]], axis=3)                                   # [rows, stages, 4, 24]
    bits = np.unpackbits(chunk.reshape(rows, stages * 8, 12), axis=2, bitorder="little")  # [rows, units, 96]
    fields = bits.reshape(rows, stages * 8, 16, 6)
    val6 = (fields * (1 << np.arange(6, dtype=np.uint8))).sum(axis=3).astype(np.uint8)     # field-ordered
    fp6 = val6[:, :, _unit_field_order()]                                                # code-ordered
    mag_bits = fp6 & 31
    lut = np.full(32, -1, dtype=np.int16)
    for bits_, mag in _E2M3_VAL.items():
        lut[bits_] = mag
    mag = lut[mag_bits]
    assert (mag >= 0).all(), "a 6-bit field is not the E2M3 code of an integer in [-7, 7]"
    codes = np.where(fp6 & 32, -mag, mag).astype(np.int8).reshape(rows, stages * 128)
    assert not codes[:, K:].any(), "K padding of a code matrix must be zero codes"
    return np.ascontiguousarray(codes[:, :K])


def unpack_host(buf, rows: int, K: int) -> np.ndarray:
    """4-bit code matrix as the library stores it (tensor or array) -> int8 codes [rows, K]."""
    if isinstance(buf, torch.Tensor):
        buf = buf.cpu().numpy()
    return decode_e2m3(buf, rows, K)


def unpack_host8(buf, rows: int, K: int) -> np.ndarray:
    """8-bit code matrix as the library stores it -> int8 codes [rows, K]."""
    if isinstance(buf, torch.Tensor):
        buf = buf.cpu().numpy()
    return from_panels(buf, rows, K).view(np.int8)


def codes4_to_dev(codes: np.ndarray) -> torch.Tensor:
    """int8 codes [rows, K] in [-7, 7] -> 4-bit code matrix on the GPU, in the library's layout."""
    return torch.from_numpy(encode_e2m3(codes)).cuda()


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
