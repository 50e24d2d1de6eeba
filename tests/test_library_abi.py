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
    return sorted(set(re.findall(r"\b(hora_[a-z0-9_]+)\s*\(", text)))


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
    for code in range(-6, 0):
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
    # the depth bound: a budget that would force some prompt beyond HORA_MAX_DEPTH = 2^20 additional
    # rollouts is refused on the host (no kernel may run a serial chain of that length)
    depth = 1 << 20
    assert alloc(1, 4, fake, 1.0, 1.0, 2_000_000_000, 0, 0, fake, None, None, 0, None, status, fake, 1 << 20, None) == UNSUPPORTED
    for method in (0, 1, 2):
        assert alloc(3, 4, fake, 1.0, 1.0, 3 * depth + 1, 0, method, fake, None, None, 0, None, status, fake,
                     1 << 20, None) == UNSUPPORTED
    assert lib.hora_allocate_posterior(3, 4, fake, fake, 3 * depth + 1, 0, fake, None, None, 0, None, status, fake,
                                       1 << 24, None) == UNSUPPORTED
    assert lib.hora_allocate_baseline(3, 4, fake, 1.0, 1.0, 3 * depth + 1, 0, 1, fake, None, None, 0, None, status,
                                      fake, 1 << 24, None) == UNSUPPORTED
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
    rows = (4 * 170856406 + 12 + 8191) // 8192          # 8 KiB rows, worst-case alignment skew
    assert need % 256 == 0 and 96 * rows <= need <= 96 * (rows + 64) + 512        # a short (32 B) and a wide (64 B) descriptor per row
    assert lib.hora_token_broadcast_workspace_bytes(0, 0) >= 256
    assert lib.hora_token_broadcast_workspace_bytes(-1, 0) == 0
    mg = lib.hora_marginal_gains
    assert mg(-1, fake, fake, 4, fake, None, None) == INVALID
    assert mg(0, fake, fake, 4, fake, None, None) == 0


def test_host_argument_validation_of_the_later_entry_points(lib):
    INVALID, INFEASIBLE, WORKSPACE, UNSUPPORTED = -1, -2, -3, -6
    fake = ctypes.c_void_p(0x1000)
    status = ctypes.c_void_p(0x2000)
    odd = ctypes.c_void_p(0x1004)            # 4-byte aligned only
    big = 1 << 24
    # sharded allocation
    sh = lib.hora_allocate_sharded
    assert sh(-1, 4, fake, 1.0, 1.0, 2, fake, fake, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert sh(8, 4, fake, 1.0, -1.0, 2, fake, fake, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert sh(8, 4, fake, 1.0, 1.0, 0, fake, fake, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert sh(8, 4, fake, 1.0, 1.0, 2, None, fake, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert sh(8, 4, fake, 1.0, 1.0, 2, odd, fake, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert sh(8, 4, fake, 1.0, 1.0, 2, fake, fake, 0, fake, None, fake, 5, None, status, fake, big, None) == INVALID
    assert sh(1 << 29, 4, fake, 1.0, 1.0, 2, fake, fake, 0, fake, None, fake, 0, None, status, fake, big, None) == INVALID
    assert sh(8, 4, fake, 1.0, 1.0, 2, fake, fake, 0, fake, None, None, 0, None, None, fake, big, None) == INVALID
    assert sh(8, 4, fake, 1.0, 1.0, 2, fake, fake, 0, fake, None, None, 0, None, status, None, 0, None) == WORKSPACE
    assert sh(8, 4, fake, 1.0, 1.0, 2, fake, fake, 0, fake, None, None, 0, None, status, fake, 64, None) == WORKSPACE
    assert sh(8, 4, fake, 1.0, 1.0, 1 << 32, fake, fake, 0, fake, None, None, 0, None, status, fake, big, None) == UNSUPPORTED
    prev = 0
    for shards in (0, 1, 4, 8192, 8193, 1 << 20):
        b = lib.hora_allocate_sharded_workspace_bytes(shards)
        assert b % 256 == 0 and b >= prev and b > 0
        prev = b
    assert lib.hora_allocate_sharded_workspace_bytes(-1) == 0
    # baseline rules
    base = lib.hora_allocate_baseline
    assert base(8, 4, fake, 1.0, 1.0, 8, 0, 7, fake, None, None, 0, None, status, fake, big, None) == INVALID      # rule
    assert base(8, 64, fake, 1.0, 1.0, 8, 0, 0, fake, None, None, 0, None, status, fake, big, None) == UNSUPPORTED # g0
    assert base(8, 4, fake, 1.0, 1.0, 25, 3, 0, fake, None, None, 0, None, status, fake, big, None) == INFEASIBLE
    assert base(0, 4, fake, 1.0, 1.0, 1, 0, 1, fake, None, None, 0, None, status, fake, big, None) == INFEASIBLE
    assert base(8, 4, fake, 1.0, 1.0, 8, 0, 1, fake, None, None, 0, None, status, fake, 16, None) == WORKSPACE
    # per-prompt posteriors
    post = lib.hora_allocate_posterior
    assert post(8, 4, None, fake, 8, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert post(8, 4, odd, fake, 8, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert post(8, 4, fake, fake, -1, 0, fake, None, None, 0, None, status, fake, big, None) == INVALID
    assert post(8, 4, fake, fake, 1 << 53, 4, fake, None, None, 0, None, status, fake, big, None) == UNSUPPORTED
    assert post(8, 4, fake, fake, 8, 0, fake, None, None, 0, None, status, fake, 16, None) == WORKSPACE
    # loss weights
    wt = lib.hora_response_weights
    assert wt(4, fake, 0, 16, fake, 1, 0.0, fake, 0, None, None) == INVALID                  # status word
    assert wt(4, fake, 3, 16, fake, 1, 0.0, fake, 0, status, None) == INVALID                # offset type
    assert wt(4, fake, 0, 16, fake, 1, float("nan"), fake, 0, status, None) == INVALID       # length constant
    assert wt(4, fake, 0, 16, odd, 1, 0.0, fake, 0, status, None) == INVALID                 # int64 offsets misaligned
    assert wt(0, fake, 0, 16, fake, 1, 0.0, fake, 0, status, None) == INVALID                # responses without groups
    assert wt(0, fake, 0, 0, fake, 1, 0.0, fake, 0, status, None) == 0
    # Pass@K (ks is read on the host)
    pk = lib.hora_pass_at_k
    ks = (ctypes.c_int32 * 3)(1, 8, 64)
    bad_ks = (ctypes.c_int32 * 3)(1, 0, 64)
    need = lib.hora_pass_at_k_workspace_bytes(500, 3)
    assert need > 0 and need % 256 == 0
    assert lib.hora_pass_at_k_workspace_bytes(500, 65) == 0
    assert pk(500, fake, fake, 0, ks, None, fake, status, fake, need, None) == 0               # no K: nothing to do
    assert pk(500, fake, fake, 65, ks, None, fake, status, fake, need, None) == UNSUPPORTED
    assert pk(500, fake, fake, 3, None, None, fake, status, fake, need, None) == INVALID
    assert pk(500, fake, fake, 3, bad_ks, None, fake, status, fake, need, None) == INVALID
    assert pk(500, None, fake, 3, ks, None, fake, status, fake, need, None) == INVALID
    assert pk(500, fake, fake, 3, ks, None, fake, status, None, 0, None) == WORKSPACE
    assert pk(500, fake, fake, 3, ks, None, fake, status, fake, 8, None) == WORKSPACE


def test_binding_refuses_to_run_without_the_library(tmp_path):
    from paper_2605_07114_amd import hora
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        hora.load_library(str(tmp_path / "libhora.so"))


def test_prepared_refuses_what_the_binding_refuses():
    """hora.prepared runs the binding's own checks (here: a host tensor where a device buffer
    is expected) and leaves the module ready for the next call."""
    import torch
    from paper_2605_07114_amd import hora
    c = torch.zeros(8, dtype=torch.int32)
    delta = torch.zeros(8, dtype=torch.int32)
    status = torch.zeros(1, dtype=torch.int32)
    ws = torch.zeros(1024, dtype=torch.uint8)
    for _ in range(2):
        with pytest.raises(ValueError):
            hora.prepared(hora.hora_allocate, c, 4, 8, delta, status, ws)
    with pytest.raises(ValueError):
        hora.prepared(hora.hora_allocate_workspace_bytes, 8, 4)   # makes no launching call
