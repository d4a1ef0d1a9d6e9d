"""CPU checks of the test-side codec for the library's 4-bit code matrices (tests/gpu_util.py): the E2M3 table
against the format's definition, and encode/decode against each other and against hand-placed bytes."""
import numpy as np

from gpu_util import _E2M3_MAG, decode_e2m3, encode_e2m3


def test_e2m3_table_is_the_format():
    # FP6 E2M3: 1 sign, 2 exponent, 3 mantissa bits, bias 1; exponent 0 is subnormal (mantissa / 8)
    for q in range(8):
        bits = int(_E2M3_MAG[q])
        e, m = bits >> 3, bits & 7
        value = m / 8.0 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 1)
        assert value == q, (q, bits)
    assert len(set(int(b) for b in _E2M3_MAG)) == 8 and max(int(b) for b in _E2M3_MAG) < 32


def test_roundtrip_and_sizes():
    rng = np.random.default_rng(0)
    for rows, K in ((1, 32), (37, 96), (32, 128), (33, 160), (5, 3072)):
        codes = rng.integers(-7, 8, size=(rows, K)).astype(np.int8)
        buf = encode_e2m3(codes)
        assert buf.size == -(-rows // 32) * -(-K // 128) * 3072
        assert np.array_equal(decode_e2m3(buf, rows, K), codes)


def test_single_code_lands_where_the_header_says():
    # row 9, code 37 = unit 2 (even: first unit of chunk 1), element 5 -> field 2 * 5 + 0 = 10 -> bits 60..65 of
    # the unit, i.e. bit 4 of byte 7 upward; A part of chunk 1 of row 9: 9 * 64 + ((1 ^ (((9 >> 1) ^ (9 >> 3)) & 3)) * 16)
    codes = np.zeros((32, 128), dtype=np.int8)
    codes[9, 37] = -3                       # E2M3: sign 1, exponent 2, mantissa 4 -> 0b110100
    buf = encode_e2m3(codes)
    a_part = 9 * 64 + ((1 ^ (((9 >> 1) ^ (9 >> 3)) & 3)) * 16)
    expect = np.zeros(3072, dtype=np.uint8)
    field = 0b110100 << 60                  # within the unit's 96-bit string
    expect[a_part:a_part + 12] = np.frombuffer(int(field).to_bytes(12, "little"), dtype=np.uint8)
    assert np.array_equal(buf, expect)
    # an odd unit: row 20, code 16 * 7 + 12 = 124 (unit 7: second unit of chunk 3), element 12 -> field 2 * 4 + 1 = 9
    codes[:] = 0
    codes[20, 124] = 7                      # 0b011110
    buf = encode_e2m3(codes)
    unit_bytes = np.frombuffer(int(0b011110 << 54).to_bytes(12, "little"), dtype=np.uint8)
    a_part = 20 * 64 + ((3 ^ (((20 >> 1) ^ (20 >> 3)) & 3)) * 16)
    b_part = 2048 + 20 * 32 + ((3 ^ ((20 >> 3) & 3)) * 8)
    expect = np.zeros(3072, dtype=np.uint8)
    expect[a_part + 12:a_part + 16] = unit_bytes[:4]     # an odd unit's first dword closes the chunk's A part
    expect[b_part:b_part + 8] = unit_bytes[4:]
    assert np.array_equal(buf, expect)
