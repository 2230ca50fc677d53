"""The C-ABI library loads, exports every function the header declares, and
rejects invalid arguments before touching a device.  CPU only: no call here
reaches a GPU."""

import ctypes as C
import os
import re

import pytest

from paper_1603_06809_amd import vbcast as V

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "vbcast.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:vbcast|bcast)_\w+)\s*\(", text)))


def test_library_is_built():
    assert os.path.exists(V.LIB_PATH), "build the library first (see __graft_entry__.build)"


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert "bcast_plan" in names and "bcast_run" in names and "vbcast_comm_create" in names
    lib = V.lib()
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(V.EXPORTS) == names


def test_plan_info_struct_matches_header():
    text = open(HEADER).read()
    body = re.search(r"typedef struct vbcast_plan_info \{(.*?)\} vbcast_plan_info;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        ctype, names = decl.split(None, 1)
        fields += [(n.strip(), ctype) for n in names.split(",")]
    want = {"int32_t": C.c_int32, "uint64_t": C.c_uint64}
    assert [(n, want[t]) for n, t in fields] == [(n, t) for n, t in V.PlanInfo._fields_]


def test_invalid_arguments_are_rejected_without_a_device():
    lib = V.lib()
    h = C.c_void_p()
    one = (C.c_void_p * 1)(0x1000)
    assert lib.vbcast_comm_create(0, one, 16, C.byref(h)) == V.ERR_ARG
    assert lib.vbcast_comm_create(-3, one, 16, C.byref(h)) == V.ERR_ARG
    assert lib.vbcast_comm_create(8193, one, 16, C.byref(h)) == V.ERR_ARG
    assert lib.vbcast_comm_create(1, None, 16, C.byref(h)) == V.ERR_ARG
    assert lib.vbcast_comm_create(1, one, 16, None) == V.ERR_ARG
    null = (C.c_void_p * 1)(None)
    assert lib.vbcast_comm_create(1, null, 16, C.byref(h)) == V.ERR_ARG
    odd = (C.c_void_p * 2)(0x1000, 0x2008)
    assert lib.vbcast_comm_create(2, odd, 16, C.byref(h)) == V.ERR_ALIGN
    assert not h.value
    assert lib.vbcast_comm_destroy(None) == V.ERR_ARG
    assert lib.bcast_plan(None, 1, 1, 0, 0, None, C.byref(h)) == V.ERR_ARG
    assert lib.bcast_plan(None, 1, 1, 0, 0, None, None) == V.ERR_ARG
    assert lib.bcast_run(None, None) == V.ERR_ARG
    assert lib.bcast_run_steps(None, 0, 0, None) == V.ERR_ARG
    assert lib.bcast_plan_info(None, None) == V.ERR_ARG
    assert lib.bcast_plan_destroy(None) == V.ERR_ARG
    assert lib.vbcast_set_tile_bytes(1000) == V.ERR_ARG
    assert lib.vbcast_set_tile_bytes(1 << 20) == V.ERR_ARG
    assert lib.vbcast_set_tile_bytes(16384) == V.SUCCESS
    assert lib.vbcast_set_chain_slab_bytes(3000) == V.ERR_ARG
    assert lib.vbcast_set_chain_slab_bytes(8192) == V.SUCCESS
    assert lib.vbcast_set_ring_executor(7) == V.ERR_ARG
    assert lib.vbcast_set_chain_schedule(3) == V.ERR_ARG
    assert lib.vbcast_set_chain_schedule(V.CHAIN_AUTO) == V.SUCCESS
    assert lib.vbcast_set_chain_workgroups_per_cu(0) == V.ERR_ARG
    assert lib.bcast_run_timed(None, None, None) == V.ERR_ARG
    assert lib.bcast_plan_census(None, 24, None, None) == V.ERR_ARG
    assert lib.bcast_plan_export_chain(None, None, None) == V.ERR_ARG
    assert lib.bcast_plan_smp(None, 1, 1, 0, 24, 1, None, C.byref(h)) == V.ERR_ARG
    assert lib.bcast_run_smp(None, None) == V.ERR_ARG
    assert lib.bcast_run_smp_phase(None, 1, None) == V.ERR_ARG
    assert lib.bcast_smp_subplan(None, 0, None, None, None, None, None) == V.ERR_ARG
    assert lib.bcast_plan_smp_destroy(None) == V.ERR_ARG


def test_select_algo_matches_the_oracle_rule():
    """Host-only entry point: the size / process-count rule [Sec. V thresholds]."""
    from oracle import bcast_oracle as O
    names = {V.NATIVE: O.NATIVE, V.TUNED: O.TUNED, V.BINOMIAL: O.BINOMIAL, V.SCATTER_RDB: O.SCATTER_RDB}
    for P in (1, 2, 3, 8, 9, 16, 24, 64, 129, 256, 513):
        for n in (0, 1, 12287, 12288, 12289, 100_000, 524287, 524288, 524289, 30_000_000):
            for tuned in (False, True):
                assert names[V.vbcast_select_algo(n, P, tuned)] == O.select_algorithm(n, P, tuned)
    out = C.c_int()
    assert V.lib().vbcast_select_algo(10, 0, 0, C.byref(out)) == V.ERR_ARG
    assert V.lib().vbcast_select_algo(10, 4, 0, None) == V.ERR_ARG


def test_error_texts():
    for code in range(7):
        assert V.bcast_strerror(code)
    assert "unknown" in V.bcast_strerror(99)
    with pytest.raises(V.VbcastError) as e:
        V.Comm([0x1008], 16)
    assert e.value.code == V.ERR_ALIGN


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and as C++), with
    nothing but standard headers behind it."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler here")
    src = tmp_path / "use_header.c"
    src.write_text('#include "vbcast.h"\n'
                   "int main(void) { vbcast_plan_info i; vbcast_census c; (void)i; (void)c; "
                   "return VBCAST_SUCCESS; }\n")
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only"],
                ["g++", "-std=c++11", "-x", "c++", "-Wall", "-Wextra", "-Werror", "-fsyntax-only"]):
        if shutil.which(cmd[0]) is None:
            continue
        r = subprocess.run(cmd + ["-I", inc, str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_bench_runs_on_one_gpu_only():
    """bench.py --gpus N with N above 1 exits with a message that says so, before
    anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_bench_reports_counter_traffic_only_for_the_profiled_kernel(tmp_path, monkeypatch):
    """bench.py's roofline.traffic comes from the committed profile and must read
    null as soon as the kernel source, the workload or the launch shape differ from
    what the counters were taken on."""
    import hashlib
    import bench

    src = tmp_path / "kernel.hip"
    src.write_text("// kernel, first version\n")
    sha = hashlib.sha256(src.read_bytes()).hexdigest()
    prof = tmp_path / "profile.md"
    prof.write_text("text\n```traffic\nworkload=W\nunit_bytes=16384\nworkgroups_per_cu=1\n"
                    f"kernel_source_sha256={sha}\nhbm_bytes_per_launch=123456\n```\nmore text\n")
    monkeypatch.setitem(bench.PROFILES, "chains", str(prof))
    monkeypatch.setitem(bench.KERNEL_SOURCES, "chains", str(src))
    assert bench.measured_traffic("chains", "W", 16384, 1)[0] == 123456.0
    assert bench.measured_traffic("chains", "other", 16384, 1)[0] is None
    assert bench.measured_traffic("chains", "W", 8192, 1)[0] is None
    assert bench.measured_traffic("chains", "W", 16384, 2)[0] is None
    src.write_text("// kernel, changed\n")
    assert bench.measured_traffic("chains", "W", 16384, 1)[0] is None
    prof.write_text("no block here\n")
    assert bench.measured_traffic("chains", "W", 16384, 1) == (None, None)


def test_committed_profiles_match_the_kernel_sources():
    """The traffic blocks under profiles/ were taken with the kernels as they are
    now (otherwise bench.py would silently print null)."""
    import bench

    assert bench.measured_traffic("chains", "P513_n128M", 16384, 1)[0] is not None
    assert bench.measured_traffic("steps", "P513_n128M", 16384, 0)[0] is not None
