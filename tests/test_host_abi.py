"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects invalid arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2604_10152_amd as sm
from paper_2604_10152_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "specmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith(("moe_", "spec_", "specmoe_"))})


@pytest.fixture(scope="module")
def lib():
    return sm.load_library()


def test_header_and_library_agree(lib):
    declared = _declared_functions()
    assert set(declared) == set(binding.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.specmoe_abi_version() == 8


def test_status_strings(lib):
    seen = {sm.status_string(s) for s in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert sm.status_string(99) == "unknown status"


def test_workspace_query(lib):
    q = lib.moe_grouped_swiglu_workspace_bytes
    assert q(0, 8, 8, 1, 0) > 0
    assert q(32, 256, 512, 8, 0) >= 32 * 512 * 4
    assert q(4096, 4096, 14336, 8, 1) >= 4096 * 14336 * 2
    assert q(4096, 4096, 14336, 8, 1) % 256 == 0
    assert q(-1, 8, 8, 1, 0) == 0 and q(1, 8, 8, 1, 7) == 0 and q(1, 0, 8, 1, 0) == 0


P = ctypes.c_void_p(0x1000)   # never dereferenced: validation fails first in every call below
N = None


def test_static_scratch_validation(lib):
    f = lib.moe_grouped_swiglu_static
    assert f(P, P, P, P, P, 8, 64, 64, 2, 7, P, N) == 3                  # dtype
    assert f(P, P, P, P, P, 8, 64, 60, 2, 1, P, N) == 2                  # d_ff % 64 in bf16
    assert f(N, P, P, P, P, 8, 64, 64, 2, 1, P, N) == 1                  # NULL
    assert f(P, P, P, P, P, 8193, 64, 1024, 2, 1, P, N) == 4             # beyond the 16 MiB scratch
    assert f(P, P, P, P, P, 4097, 64, 1024, 2, 0, P, N) == 4             # same, fp32
    assert f(P, P, P, P, P, 0, 64, 64, 2, 1, P, N) == 0                  # nothing to do


def test_packed_entry_points_validation(lib):
    pw, hb = lib.moe_pack_weights, lib.moe_packed_h_bytes
    assert pw(P, 2, 64, 64, 0, ctypes.c_void_p(0x100000), N) == 3        # fp32 is not packed
    assert pw(P, 2, 60, 64, 1, ctypes.c_void_p(0x100000), N) == 2        # rows % 16
    assert pw(P, 2, 64, 48, 1, ctypes.c_void_p(0x100000), N) == 2        # cols % 32
    assert pw(P, 2, 64, 64, 1, P, N) == 2                                # in place
    assert pw(N, 2, 64, 64, 1, P, N) == 1
    assert hb(4096, 14336, 8) == (4096 // 16 + 8) * 16 * 14336 * 2
    assert hb(-1, 64, 1) == 0
    up, down = lib.moe_expert_up_swiglu_gather_packed, lib.moe_expert_down_packed
    assert up(P, N, 0, 1, P, P, P, 64, 64, 64, 2, 0, P, 1 << 30, N, 0, N) == 3  # bf16 only
    assert up(P, N, 0, 1, P, P, P, 64, 64, 64, 2, 1, P, 16, N, 0, N) == 4       # h too small
    assert up(P, P, 8, 2, P, P, P, 64, 64, 64, 2, 1, P, 1 << 30, N, 0, N) == 2  # n_rows > T*k
    assert up(P, N, 0, 1, P, P, P, 64, 64, 64, 2, 1, P, 1 << 30, P, 16, N) == 4  # x workspace too small
    assert down(P, P, P, 64, 64, 64, 2, 0, P, N) == 3
    assert down(N, P, P, 64, 64, 64, 2, 1, P, N) == 1
    rows, upp = lib.moe_permute_rows_packed, lib.moe_expert_up_swiglu_packed
    big = 1 << 30
    assert rows(P, N, 0, 1, P, 64, 64, 2, 0, P, big, N) == 3             # bf16 only
    assert rows(P, N, 0, 1, P, 64, 60, 2, 1, P, big, N) == 2             # d_model % 64
    assert rows(P, P, 8, 2, P, 64, 64, 2, 1, P, big, N) == 2             # n_rows > T*k
    assert rows(P, N, 0, 1, P, 64, 64, 2, 1, P, 16, N) == 4              # x_packed too small
    assert rows(P, N, 0, 1, N, 64, 64, 2, 1, P, big, N) == 1
    assert rows(N, N, 0, 1, N, 0, 64, 2, 1, N, 0, N) == 0                # nothing to do
    assert upp(P, big, P, P, P, 64, 64, 64, 2, 0, P, big, 0, N) == 3
    assert upp(P, 16, P, P, P, 64, 64, 64, 2, 1, P, big, 0, N) == 4      # x_packed too small
    assert upp(P, big, P, P, P, 64, 64, 64, 2, 1, P, 16, 0, N) == 4      # h_packed too small
    assert upp(P, big, P, P, P, 64, 64, 64, 2, 1, P, 64 * 64 * 2 - 1, 1, N) == 4   # row-major h too small
    assert upp(N, big, P, P, P, 64, 64, 64, 2, 1, P, big, 0, N) == 1
    assert upp(P, big, P, P, P, 64, 64, 100, 2, 1, P, big, 0, N) == 2


def test_route_validation(lib):
    f = lib.moe_route_topk
    assert f(P, P, N, 4, 8, 8, 2, 1, 5, P, P, N) == 3            # dtype
    assert f(P, P, N, 4, 8, 8, 9, 1, 0, P, P, N) == 2            # k > E
    assert f(P, P, N, 4, 8, 0, 1, 1, 0, P, P, N) == 2            # E < 1
    assert f(P, P, N, 4, 8, 2000, 1, 1, 0, P, P, N) == 2         # E too large
    assert f(P, P, N, -1, 8, 8, 2, 1, 0, P, P, N) == 2           # T < 0
    assert f(P, P, N, 4, 0, 8, 2, 1, 0, P, P, N) == 2            # d < 1
    assert f(P, P, N, 2 ** 30, 8, 8, 8, 1, 0, P, P, N) == 2      # T*k overflows
    assert f(N, P, N, 4, 8, 8, 2, 1, 0, P, P, N) == 1            # null x
    assert f(P, P, N, 4, 8, 8, 2, 1, 0, N, P, N) == 1            # null idx
    assert f(N, N, N, 0, 8, 8, 2, 1, 0, N, N, N) == 0            # T = 0 is legal


def test_permute_validation(lib):
    f = lib.moe_permute
    assert f(P, P, 4, 8, 8, 2, 9, P, P, P, P, N) == 3
    assert f(P, P, 4, 8, 8, 9, 0, P, P, P, P, N) == 2
    assert f(P, P, 4, 8, 8, 2, 0, P, N, P, P, N) == 1            # offsets required
    assert f(P, N, 4, 8, 8, 2, 0, P, P, P, P, N) == 1
    assert f(N, P, 4, 8, 8, 2, 0, P, P, P, P, N) == 1            # x_perm wanted but x missing


def test_grouped_validation(lib):
    f = lib.moe_grouped_swiglu
    big = 1 << 40
    assert f(P, P, P, P, P, 8, 64, 64, 2, 4, P, P, big, N) == 3
    assert f(P, P, P, P, P, -8, 64, 64, 2, 0, P, P, big, N) == 2
    assert f(P, P, P, P, P, 8, 60, 64, 2, 1, P, P, big, N) == 2   # bf16 needs d % 64 == 0
    assert f(P, P, P, P, P, 8, 64, 100, 2, 1, P, P, big, N) == 2  # bf16 needs f % 64 == 0
    assert f(N, P, P, P, P, 8, 64, 64, 2, 1, P, P, big, N) == 1
    assert f(P, P, P, P, P, 8, 64, 64, 2, 1, P, N, big, N) == 1
    assert f(P, P, P, P, P, 8, 64, 64, 2, 1, P, P, 16, N) == 4    # workspace too small
    assert f(P, P, P, P, P, 8, 64, 64, 2, 1, P, ctypes.c_void_p(0x1010), big, N) == 4  # misaligned
    assert f(N, N, N, N, N, 0, 64, 64, 2, 1, N, N, 0, N) == 0     # no rows: nothing to do


def test_gather_up_validation(lib):
    f = lib.moe_expert_up_swiglu_gather
    assert f(P, P, 4, 2, P, P, P, 8, 64, 64, 2, 7, P, N) == 3
    assert f(P, P, 4, 2, P, P, P, 9, 64, 64, 2, 1, P, N) == 2            # n_rows > T*k
    assert f(P, P, 4, 0, P, P, P, 8, 64, 64, 2, 1, P, N) == 2            # k < 1
    assert f(P, P, 2 ** 20, 2, P, P, P, 8, 4096, 64, 2, 1, P, N) == 2    # 32-bit row offsets
    assert f(N, P, 4, 2, P, P, P, 8, 64, 64, 2, 1, P, N) == 1
    assert f(P, N, 4, 2, P, P, P, 8, 64, 64, 2, 1, P, N) == 1
    assert f(N, N, 4, 2, N, N, N, 0, 64, 64, 2, 1, N, N) == 0


def test_combine_accept_rmsnorm_validation(lib):
    c = lib.moe_combine
    assert c(P, P, P, N, 4, 8, 2, 3, P, N) == 3
    assert c(P, P, P, N, 4, 8, 0, 0, P, N) == 2
    assert c(P, P, P, N, 4, 8, 2, 0, N, N) == 1
    assert c(N, N, N, N, 0, 8, 2, 0, N, N) == 0
    a = lib.spec_accept
    assert a(P, P, -1, 3, P, P, N) == 2
    assert a(P, P, 4, -3, P, P, N) == 2
    assert a(N, P, 4, 3, P, P, N) == 1
    assert a(P, P, 4, 3, N, P, N) == 1
    assert a(N, N, 0, 3, N, N, N) == 0
    h = lib.moe_hot_experts
    assert h(P, 0, 0, P, N, N) == 2
    assert h(P, 8, 9, P, N, N) == 2
    assert h(N, 8, 2, P, N, N) == 1
    assert h(P, 8, 2, N, N, N) == 1
    assert h(N, 8, 0, N, N, N) == 0
    r = lib.moe_rmsnorm
    assert r(P, P, 4, 8, 1e-5, 2, P, N) == 3
    assert r(P, P, 4, 8, -1.0, 0, P, N) == 2
    assert r(P, N, 4, 8, 1e-5, 0, P, N) == 1


def test_speculation_phase_validation(lib):
    q = lib.moe_affinity_table_workspace_bytes
    assert q(0) == 0 and q(2000) == 0
    assert q(8) == 1 * 1024 * 64 * 8 and q(9) == 3 * 1024 * 64 * 8 and q(64) == 36 * 1024 * 64 * 8
    P16 = ctypes.c_void_p(0x1000)
    a = lib.moe_affinity_table
    assert a(P16, P16, P16, 8, 64, 64, 7, P, P, 1 << 30, N) == 3                 # dtype
    assert a(P16, P16, P16, 0, 64, 64, 1, P, P, 1 << 30, N) == 2                 # E < 1
    assert a(P16, P16, P16, 8, 3, 5, 1, P, P, 1 << 30, N) == 2                   # 30 bytes per matrix
    assert a(ctypes.c_void_p(0x1004), P16, P16, 8, 64, 64, 1, P, P, 1 << 30, N) == 2   # alignment
    assert a(N, P16, P16, 8, 64, 64, 1, P, P, 1 << 30, N) == 1
    assert a(P16, P16, P16, 8, 64, 64, 1, P, N, 1 << 30, N) == 1
    assert a(P16, P16, P16, 8, 64, 64, 1, P, P, 100, N) == 4                     # workspace
    n = lib.moe_nearest_draft_expert
    assert n(P, 8, P, 0, P, N) == 2 and n(P, 8, P, 9, P, N) == 2 and n(P, 0, P, 1, P, N) == 2
    assert n(N, 8, P, 2, P, N) == 1 and n(P, 8, N, 2, P, N) == 1 and n(P, 8, P, 2, N, N) == 1
    r = lib.moe_route_topk_draft
    assert r(P, P, N, 4, 8, 8, 2, 1, 5, P, P, P, N) == 3
    assert r(P, P, N, 4, 8, 8, 9, 1, 0, P, P, P, N) == 2
    assert r(P, P, N, 4, 8, 8, 2, 1, 0, N, P, P, N) == 1                         # remap missing
    assert r(N, N, N, 0, 8, 8, 2, 1, 0, P, N, N, N) == 0


def test_sampling_and_reporting_validation(lib):
    s = lib.spec_accept_sample
    assert s(P, P, P, P, P, -1, 3, 10, P, P, N) == 2
    assert s(P, P, P, P, P, 4, 65, 10, P, P, N) == 2                             # gamma > 64
    assert s(P, P, P, P, P, 4, 3, 0, P, P, N) == 2
    assert s(N, P, P, P, P, 4, 3, 10, P, P, N) == 1
    assert s(P, P, N, P, P, 4, 3, 10, P, P, N) == 1
    assert s(P, P, P, P, P, 4, 3, 10, N, P, N) == 1
    assert s(N, N, N, N, N, 0, 3, 10, N, N, N) == 0
    g = lib.spec_greedy_tokens
    assert g(P, 4, 10, 3, P, N) == 3 and g(P, -1, 10, 0, P, N) == 2 and g(P, 4, 0, 0, P, N) == 2
    assert g(N, 4, 10, 0, P, N) == 1 and g(P, 4, 10, 0, N, N) == 1 and g(N, 0, 10, 0, N, N) == 0
    b = lib.moe_active_expert_bytes
    assert b(P, 0, 10, P, N) == 2 and b(P, 8, -1, P, N) == 2
    assert b(N, 8, 10, P, N) == 1 and b(P, 8, 10, N, N) == 1


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(4, 8)
    with pytest.raises(TypeError):
        sm.moe_route_topk(x, torch.zeros(2, 8), None, 1, True, torch.zeros(4, 1, dtype=torch.int32),
                          torch.zeros(4, 1), stream=object())
