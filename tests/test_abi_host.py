"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and argument
validation returns the documented status before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "convrot.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2512_03673_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2512_03673_amd import build
        build.build(verbose=False)
    return binding.load()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conv(?:rot|linear4bit|linear8bit)_\w+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    from paper_2512_03673_amd import binding
    names = declared_symbols()
    assert len(names) == 22
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert getattr(lib, n) is not None


def test_size_queries_and_strings(lib):
    from paper_2512_03673_amd import binding as b
    assert b.version() == 500
    # 4-bit code matrices: 3 KB blocks of 32 rows x 128 codes (6 bits per code), rows and K padded up to whole blocks
    assert b.packed_bytes(4608, 3072) == 4608 * 3072 * 3 // 4
    assert b.packed_bytes(37, 96) == 2 * 1 * 3072 and b.packed_bytes(3, 32) == 3072
    assert b.packed_bytes(32, 128) == 3072 and b.packed_bytes(33, 160) == 2 * 2 * 3072
    assert b.packed_bytes(0, 32) == 0
    assert b.packed_bytes(-1, 32) == 0 and b.packed_bytes(4, 33) == 0
    # 8-bit code matrices: 1 KB panels of 16 rows x 64 bytes
    assert b.packed_bytes8(37, 96) == 3 * 2 * 1024 and b.packed_bytes8(4608, 3072) == 4608 * 3072
    # code matrix + scales rounded up to 256 B
    assert b.workspace_bytes(4608, 3072) == 4608 * 3072 * 3 // 4 + 4608 * 4
    assert b.workspace_bytes(3, 32) == 3072 + 256
    assert b.workspace_bytes(0, 32) == 0
    assert b.workspace_bytes8(4608, 3072) == 4608 * 3072 + 4608 * 4
    assert b.workspace_bytes8(3, 32) == 1024 + 256
    assert "clang" in b.build_info() and "HIP" in b.build_info()
    assert b.status_string(0) == "ok"
    assert "group" in b.status_string(-3)
    assert b.status_string(-99) == "unknown status"


def test_gemm_tile_choice(lib):
    from paper_2512_03673_amd import binding as b
    # up to 256 tiles of either shape the smaller tile (256 x 128) has less work per block
    assert b.gemm_tile_rows(256, 1024) == 256 and b.gemm_tile_rows(4608, 3072) == 256
    # 256 square tiles against 288 of the other shape: one block per compute unit against two
    assert b.gemm_tile_rows(3072, 3072) == 192 and b.gemm_tile_rows(3001, 3070) == 192
    # headline shape: 1536 square tiles (6 per unit) against 1728 (7 per unit)
    assert b.gemm_tile_rows(4608, 12288) == 192
    assert b.gemm_tile_rows(-1, 5) == 0 and b.gemm_tile_rows(5, -1) == 0


def test_argument_validation_without_a_device(lib):
    # fake, suitably aligned addresses: validation must reject before touching them
    A = 0x10000
    f = lib.convrot_rotquant_act
    assert f(None, 4, 1024, 16, A, A, None) == -1
    assert f(A, 4, 1024, 16, None, A, None) == -1
    assert f(A, 4, 1024, 16, A, None, None) == -1
    assert f(A, 4, 1024, 8, A, A, None) == -3
    assert f(A, -1, 1024, 16, A, A, None) == -2
    assert f(A, 4, 0, 16, A, A, None) == -2
    assert f(A, 4, 1040, 16, A, A, None) == -2          # K % 32 != 0
    assert f(A, 4, 96, 64, A, A, None) == -2            # K % g != 0
    assert f(A, 4, 131072, 16, A, A, None) == -2        # K > CONVROT_MAX_K
    assert f(A + 8, 4, 1024, 16, A, A, None) == -4
    assert f(A, 4, 1024, 16, A + 4, A, None) == -4
    assert f(A, 4, 1024, 16, A, A + 2, None) == -4
    p = lib.convrot_prepare_weight
    assert p(None, 4, 1024, 16, A, A, None) == -1
    assert p(A, 4, 1024, 3, A, A, None) == -3
    g = lib.convrot_w4a4_gemm_dequant
    assert g(None, A, A, A, None, 4, 4, 1024, A, None) == -1
    assert g(A, None, A, A, None, 4, 4, 1024, A, None) == -1
    assert g(A, A, A, A, None, 4, -4, 1024, A, None) == -2
    assert g(A, A, A, A, A, 4, 4, 1000, A, None) == -2
    assert g(A, A, A + 1, A, None, 4, 4, 1024, A, None) == -4
    assert g(A, A, A, A, A + 1, 4, 4, 1024, A, None) == -4      # bias is bf16: 2-byte aligned
    r = lib.convrot_w4a4_gemm_i32
    assert r(A, A, 4, 4, 1024, None, None) == -1
    assert r(A, A, 4, 4, 48, A, None) == -2
    fw = lib.convlinear4bit_forward
    assert fw(A, A, A, None, 4, 4, 1024, 16, A, None, 1 << 20, None) == -1
    assert fw(A, A, A, None, 4, 4, 1024, 5, A, A, 1 << 20, None) == -3
    assert fw(A, A, A, A, 4, 4, 1024, 16, A, A + 16, 1 << 20, None) == -4
    assert fw(A, A, A, A + 1, 4, 4, 1024, 16, A, A, 1 << 20, None) == -4
    assert fw(A, A, A, None, 4, 4, 1024, 16, A, A, 100, None) == -5
    # the variant with the static workspace: same checks, the size limit instead of the workspace check, all on the host
    fn = lib.convlinear4bit_forward_noalloc
    assert fn(None, A, A, None, 4, 4, 1024, 16, A, None) == -1
    assert fn(A, A, A, None, 4, 4, 1024, 5, A, None) == -3
    assert fn(A, A, A, A + 1, 4, 4, 1024, 16, A, None) == -4
    assert fn(A, A, A, None, 4, 4, 1040, 16, A, None) == -2
    assert fn(A, A, A, None, 16896, 4, 12288, 16, A, None) == -5      # 156 MB of codes: beyond the 64 MiB array
    assert fn(A, A, A, None, 0, 4, 1024, 16, A, None) == 0
    # W8A8 variant: same validation
    f8, g8, fw8 = lib.convrot_rotquant_act8, lib.convrot_w8a8_gemm_dequant, lib.convlinear8bit_forward
    assert f8(A, 4, 48, 16, A, A, None) == -2            # K % 32 != 0
    assert f8(None, 4, 1024, 16, A, A, None) == -1
    assert lib.convrot_prepare_weight8(A, 4, 1024, 5, A, A, None) == -3
    assert g8(A, A, A, A, None, 4, 4, 48, A, None) == -2
    assert g8(A, None, A, A, None, 4, 4, 1024, A, None) == -1
    assert lib.convrot_w8a8_gemm_i32(A, A, 4, 4, 1024, None, None) == -1
    assert fw8(A, A, A, None, 4, 4, 1024, 16, A, A, 100, None) == -5
    assert fw8(A, A, A, None, 4, 4, 1040, 16, A, A, 1 << 20, None) == -2
    assert g8(A, A, A, A, None, 0, 4, 1024, A, None) == 0
    u = lib.convrot_unpack_codes
    assert u(None, 4, 1024, A, None) == -1 and u(A, 4, 1000, A, None) == -2 and u(A, 4, 1024, A + 8, None) == -4
    d = lib.convrot_rotated_absmax
    assert d(A, 4, 1024, 16, 3, A, None) == -3 and d(A, 4, 1024, 8, 1, A, None) == -3
    assert d(None, 4, 1024, 16, 1, A, None) == -1 and d(A, 4, 1000, 16, 1, A, None) == -2
    assert d(A, 0, 1024, 16, 2, A, None) == 0
    # empty problems are valid no-ops and launch nothing
    assert f(A, 0, 1024, 16, A, A, None) == 0
    assert g(A, A, A, A, None, 0, 4, 1024, A, None) == 0
    assert g(A, A, A, A, A, 4, 0, 1024, A, None) == 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2512_03673_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text and "oracle/" not in text, fn
