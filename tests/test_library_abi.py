"""The C-ABI library loads, exports what include/hora.h declares, and rejects bad
host arguments before touching the GPU (CPU only: no kernel is launched here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hora.h")
LIB = os.path.join(ROOT, "paper_2605_07114_amd", "libhora.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2605_07114_amd.build import build_library
        build_library()
    from paper_2605_07114_amd import hora
    return hora.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hora_[a-z_]+)\s*\(", text)))


def test_header_declares_the_entry_points():
    names = declared_functions()
    for must in ("hora_allocate", "hora_group_advantage", "hora_token_broadcast"):
        assert must in names


def test_every_declared_symbol_is_exported(lib):
    from paper_2605_07114_amd import hora
    names = declared_functions()
    assert sorted(hora.EXPORTS) == names
    for name in names:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert lib.hora_version() >= 100
    assert lib.hora_status_string(0) == b"ok"
    for code in range(-7, 0):
        assert lib.hora_status_string(code) not in (b"ok", b"unknown status")
    assert lib.hora_status_string(-99) == b"unknown status"


def test_workspace_size_is_monotone_and_aligned(lib):
    prev = 0
    for n in (0, 1, 1023, 1024, 1025, 1 << 20, (1 << 20) + 1, 1 << 26):
        b = lib.hora_allocate_workspace_bytes(n, 8)
        assert b % 256 == 0 and b >= prev and b > 0
        prev = b
    assert lib.hora_allocate_workspace_bytes(-1, 8) == 0


def test_host_argument_validation_needs_no_gpu(lib):
    INVALID, INFEASIBLE, WORKSPACE, UNSUPPORTED = -1, -2, -3, -6
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    status = ctypes.c_void_p(0x2000)
    alloc = lib.hora_allocate
    # negative sizes, missing status word, bad prior, unknown method
    assert alloc(-1, 4, fake, 1.0, 1.0, 0, 0, 0, fake, None, None, 0, None, status, fake, 1 << 20, None) == INVALID
    assert alloc(8, 4, fake, 1.0, 1.0, 8, 0, 0, fake, None, None, 0, None, None, fake, 1 << 20, None) == INVALID
    assert alloc(8, 4, fake, 0.0, 1.0, 8, 0, 0, fake, None, None, 0, None, status, fake, 1 << 20, None) == INVALID
    assert alloc(8, 4, fake, 1.0, 1.0, 8, 0, 9, fake, None, None, 0, None, status, fake, 1 << 20, None) == INVALID
    # budget that cannot be placed
    assert alloc(0, 4, fake, 1.0, 1.0, 1, 0, 0, fake, None, None, 0, None, status, fake, 1 << 20, None) == INFEASIBLE
    assert alloc(8, 4, fake, 1.0, 1.0, 25, 3, 0, fake, None, None, 0, None, status, fake, 1 << 20, None) == INFEASIBLE
    # workspace missing / too small / misaligned
    assert alloc(8, 4, fake, 1.0, 1.0, 8, 0, 0, fake, None, None, 0, None, status, None, 0, None) == WORKSPACE
    assert alloc(8, 4, fake, 1.0, 1.0, 8, 0, 0, fake, None, None, 0, None, status, fake, 16, None) == WORKSPACE
    assert alloc(8, 4, fake, 1.0, 1.0, 8, 0, 0, fake, None, None, 0, None, status, ctypes.c_void_p(0x1010),
                 1 << 20, None) == WORKSPACE
    # class method beyond its G0 limit; int32 delta overflow; int32 offsets overflow
    assert alloc(8, 64, fake, 1.0, 1.0, 8, 0, 1, fake, None, None, 0, None, status, fake, 1 << 20, None) == UNSUPPORTED
    assert alloc(8, 4, fake, 1.0, 1.0, 1 << 33, 0, 0, fake, None, None, 0, None, status, fake, 1 << 20, None) == UNSUPPORTED
    assert alloc(1 << 29, 4, fake, 1.0, 1.0, 8, 0, 0, fake, None, fake, 0, None, status, fake, 1 << 30, None) == INVALID
    # advantage / broadcast
    adv = lib.hora_group_advantage
    assert adv(4, fake, 0, 16, fake, fake, 0, 7, 0.0, 0, status, None) == INVALID       # mode
    assert adv(4, fake, 0, 16, fake, fake, 0, 0, -1.0, 0, status, None) == INVALID      # eps
    assert adv(4, fake, 0, 16, fake, fake, 0, 0, 0.0, 2, status, None) == INVALID       # ddof
    assert adv(0, fake, 0, 16, fake, fake, 0, 0, 0.0, 0, status, None) == INVALID       # responses without groups
    assert adv(0, fake, 0, 0, fake, fake, 0, 0, 0.0, 0, status, None) == 0
    bc = lib.hora_token_broadcast
    assert bc(0, fake, 0, fake, 0, fake, 0, 0, status, fake, 1 << 20, None) == 0
    assert bc(0, fake, 0, fake, 0, fake, 0, 5, status, fake, 1 << 20, None) == INVALID
    assert bc(4, fake, 0, fake, 0, fake, 1, 5, status, fake, 1 << 20, None) == INVALID        # float -> double
    assert bc(4, fake, 0, fake, 0, fake, 0, 1 << 31, status, fake, 1 << 30, None) == INVALID  # int32 offsets overflow
    assert bc(4, fake, 1, fake, 1, ctypes.c_void_p(0x1002), 0, 5, status, fake, 1 << 20, None) == INVALID  # misaligned
    assert bc(4, fake, 0, fake, 0, fake, 0, 5000, status, None, 0, None) == WORKSPACE
    assert bc(4, fake, 0, fake, 0, fake, 0, 5000, status, fake, 8, None) == WORKSPACE
    need = lib.hora_token_broadcast_workspace_bytes(170856406, 0)
    rows = (4 * 170856406 + 12 + 4095) // 4096          # 4 KiB rows, worst-case alignment skew
    assert need % 256 == 0 and 32 * (rows + 1) <= need <= 32 * (rows + 1) + 256   # one 32-byte descriptor per row
    assert lib.hora_token_broadcast_workspace_bytes(-1, 0) == 0
    mg = lib.hora_marginal_gains
    assert mg(-1, fake, fake, 4, fake, None, None) == INVALID
    assert mg(0, fake, fake, 4, fake, None, None) == 0


def test_binding_refuses_to_run_without_the_library(tmp_path):
    from paper_2605_07114_amd import hora
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        hora.load_library(str(tmp_path / "libhora.so"))
