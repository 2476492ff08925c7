"""The C-ABI library loads and exports what include/pp.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

from conftest import ROOT


@pytest.fixture(scope="module")
def libpp():
    from paper_2204_10562_amd import binding, build
    if not os.path.exists(build.LIB_PATH):
        build.build_libpp()
    return binding.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pp_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_entry_points():
    names = declared_functions()
    for want in ("pp_prefix_costs", "pp_partition_dp", "pp_schedule_makespan", "pp_best_plan"):
        assert want in names


def test_every_declared_symbol_is_exported(libpp):
    from paper_2204_10562_amd import binding
    names = declared_functions()
    assert sorted(binding.EXPORTS) == names
    for name in names:
        assert getattr(libpp, name) is not None


def test_result_struct_size():
    from paper_2204_10562_amd import binding
    assert binding.RESULT_BYTES == 8 * 3 + 4 + 4 * 64 * 2 + 4  # padded to 8-byte alignment


def test_workspace_bytes_host_function(libpp):
    from paper_2204_10562_amd import binding
    a = binding.pp_workspace_bytes(128, 8, 8, 40320)
    b = binding.pp_workspace_bytes(128, 8, 8, 2 * 40320)
    assert a > 0 and b > a and a % 256 == 0
    assert binding.pp_workspace_bytes(0, 8, 8, 1) == 0
    assert binding.pp_workspace_bytes(16, 4, 5, 1) == 0  # S > D
    assert binding.pp_workspace_bytes(4, 8, 5, 1) == 0   # S > L


def test_strerror(libpp):
    assert libpp.pp_strerror(0) == b"ok"
    for code in (-1, -2, -3):
        assert len(libpp.pp_strerror(code)) > 3


def test_host_side_argument_errors_enqueue_nothing(libpp):
    # invalid sizes / NULL required pointers are rejected before any HIP call
    z = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)  # never dereferenced: the size checks fail first
    assert libpp.pp_prefix_costs(0, 4, one, one, one, z, one, one, one, one, one, z, z) == -1
    assert libpp.pp_prefix_costs(16, 4, z, one, one, z, one, one, one, one, one, z, z) == -1
    assert libpp.pp_partition_dp(16, 4, 5, 24, one, one, one, one, one, one, one, one, 1 << 30, z, z) == -1
    assert libpp.pp_partition_dp(16, 4, 4, 23, one, one, one, one, z, one, one, one, 1 << 30, z, z) == -1
    assert libpp.pp_partition_dp(16, 4, 4, 24, one, one, one, one, z, one, one, z, 0, z, z) == -2
    assert libpp.pp_partition_dp(16, 4, 4, 24, one, one, one, one, z, one, one, one, 16, z, z) == -2
    assert libpp.pp_partition_dp(16, 4, 4, 24, one, one, one, one, z, one, one, ctypes.c_void_p(264), 1 << 30, z, z) == -2
    assert libpp.pp_schedule_makespan(16, 4, 4, 24, 0, one, one, one, one, z, one, one, z, z) == -1
    assert libpp.pp_best_plan(16, 4, 4, 24, 4, one, one, one, one, z, z, z, z, one, 1 << 30, z, z) == -1
    Ms = (ctypes.c_int32 * 2)(4, 0)
    mp = ctypes.cast(Ms, ctypes.c_void_p)
    assert libpp.pp_best_plan_multi(16, 4, 4, 24, 2, mp, one, one, one, one, z, one, z, z, one, 1 << 30, z, z) == -1  # M = 0
    assert libpp.pp_best_plan_multi(16, 4, 4, 24, 17, mp, one, one, one, one, z, one, z, z, one, 1 << 30, z, z) == -1
    assert libpp.pp_best_plan_multi(16, 4, 4, 24, 0, mp, one, one, one, one, z, one, z, z, one, 1 << 30, z, z) == -1
    assert libpp.pp_schedule_makespan_multi(16, 4, 4, 24, 2, mp, one, one, one, one, z, one, one, z, z) == -1  # M = 0
    assert libpp.pp_schedule_makespan_multi(16, 4, 4, 24, 17, mp, one, one, one, one, z, one, one, z, z) == -1
    assert libpp.pp_schedule_makespan_multi(16, 4, 4, 24, 1, mp, one, one, one, one, z, z, one, z, z) == -1   # no bounds
    # the entry point without a workspace argument: sizes beyond its array are refused
    assert libpp.pp_best_plan_static(300, 16, 16, 200000, 4, one, one, one, one, one, one, z, z, z, z) == -2
    assert libpp.pp_best_plan_static(16, 4, 4, 24, 0, one, one, one, one, z, one, z, z, z, z) == -1


def test_stage_search_and_replicated_argument_errors(libpp):
    from paper_2204_10562_amd import binding
    z = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)
    Ms = (ctypes.c_int32 * 2)(4, 8)
    mp = ctypes.cast(Ms, ctypes.c_void_p)
    # workspace sizes: the stage search needs more than the plain path, and grows with nM
    a = binding.pp_workspace_bytes(128, 8, 8, 40320)
    b1 = binding.pp_workspace_bytes_stages(128, 8, 8, 40320, 1)
    b4 = binding.pp_workspace_bytes_stages(128, 8, 8, 40320, 4)
    assert b4 > b1 > a and b4 % 256 == 0
    assert binding.pp_workspace_bytes_stages(128, 8, 8, 40320, 0) == 0
    assert binding.pp_workspace_bytes_stages(128, 8, 8, 40320, 17) == 0
    assert binding.pp_workspace_bytes_stages(128, 8, 9, 40320, 1) == 0
    assert libpp.pp_partition_dp_stages(16, 4, 5, 24, one, one, one, one, one, one, one, one, 1 << 30, z, z) == -1
    assert libpp.pp_partition_dp_stages(16, 4, 4, 24, one, one, one, one, z, one, one, one, 16, z, z) == -2
    assert libpp.pp_best_plan_stages(16, 4, 4, 24, 2, mp, one, one, one, one, z, z, z, z, one, 1 << 30, z, z) == -1  # no out
    assert libpp.pp_best_plan_stages(16, 4, 4, 24, 2, mp, one, one, one, one, z, one, z, z, one, 4096, z, z) == -2  # too small
    # replicated planner: limits on D and on what fits in LDS, all D devices per ordering
    r = binding.pp_workspace_bytes_replicated(128, 8, 40320)
    assert r > 0 and r % 256 == 0
    assert binding.pp_workspace_bytes_replicated(583, 8, 10) > 0
    assert binding.pp_workspace_bytes_replicated(584, 8, 10) == 0
    assert binding.pp_workspace_bytes_replicated(370, 16, 10) > 0
    assert binding.pp_workspace_bytes_replicated(371, 16, 10) == 0
    assert binding.pp_workspace_bytes_replicated(16, 17, 10) == 0
    args = (one,) * 6
    assert libpp.pp_plan_replicated(16, 17, 10, 4, *args, one, one, z, z, z, z, one, 1 << 30, z, z) == -1   # D > 16
    assert libpp.pp_plan_replicated(16, 4, 23, 4, *args, z, one, z, z, z, z, one, 1 << 30, z, z) == -1    # N != D!
    assert libpp.pp_plan_replicated(16, 4, 24, 0, *args, z, one, z, z, z, z, one, 1 << 30, z, z) == -1    # M = 0
    assert libpp.pp_plan_replicated(16, 4, 24, 4, *args, z, z, z, z, z, z, one, 1 << 30, z, z) == -1      # no out
    assert libpp.pp_plan_replicated(16, 4, 24, 4, *args, z, one, z, z, z, z, one, 256, z, z) == -2        # too small
    assert libpp.pp_plan_replicated(16, 4, 24, 4, *args, z, one, z, z, z, z, ctypes.c_void_p(264), 1 << 30, z, z) == -2
    # device ordering: host function
    assert libpp.pp_rdo_order(0, one, one) == -1 and libpp.pp_rdo_order(1025, one, one) == -1
    assert libpp.pp_rdo_order(4, z, one) == -1


def test_rep_result_struct_size():
    from paper_2204_10562_amd import binding
    assert binding.REP_RESULT_BYTES == 8 * 3 + 4 + 4 * 64 * 3 + 4
