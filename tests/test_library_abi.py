"""The C-ABI library loads and exports every function include/dsvt.h declares (no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2301_06051_amd", "libdsvt.so")


def _declared():
    text = open(os.path.join(ROOT, "include", "dsvt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dsvt_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_entry_points():
    names = _declared()
    for must in ("dsvt_partition", "dsvt_set_attention", "dsvt_block", "dsvt_attn_pool"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(LIB)
    for name in _declared():
        assert hasattr(lib, name), name


def test_library_exports_nothing_the_header_does_not_declare():
    """Every exported dsvt_* function is a declared one: no debug or instrumentation entry points beside the header's."""
    import subprocess
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    out = subprocess.run(["nm", "-D", "--defined-only", LIB], capture_output=True, text=True, check=True).stdout
    exported = {l.split()[-1] for l in out.splitlines() if l.split() and l.split()[-2] in ("T", "t") and l.split()[-1].startswith("dsvt_")}
    assert exported and exported <= set(_declared()), sorted(exported - set(_declared()))


def test_instrumented_library_adds_one_symbol_only():
    """The optional phase-clock build of the layer kernel is the product library plus dsvt_debug_phase_clocks."""
    import subprocess
    from paper_2301_06051_amd.build import PHASE_LIB
    if not os.path.exists(PHASE_LIB):
        pytest.skip("instrumented library not built")
    out = subprocess.run(["nm", "-D", "--defined-only", PHASE_LIB], capture_output=True, text=True, check=True).stdout
    exported = {l.split()[-1] for l in out.splitlines() if l.split() and l.split()[-2] in ("T", "t") and l.split()[-1].startswith("dsvt_")}
    assert exported - set(_declared()) == {"dsvt_debug_phase_clocks"}


def test_host_only_calls_work_without_a_gpu():
    """dsvt_partition_bound is pure host arithmetic: the set bound and a positive scratch size."""
    if not os.path.exists(LIB):
        pytest.skip("library not built")
    from paper_2301_06051_amd import binding as b
    cfg = b.part_cfg((468, 468, 1), (12, 12, 1), (6, 6, 0), 36, 1, 0)
    max_sets, max_tiles, ws = b.dsvt_partition_bound(cfg, 30000)
    assert max_sets == 30000 // 36 + 40 * 40 and ws > 0
    assert max_tiles == (30000 + 4 * max_sets) // 64 + 1 + 256
    with pytest.raises(b.DsvtError):
        b.dsvt_partition_bound(b.part_cfg((468, 468, 1), (12, 12, 1), (12, 0, 0), 36, 1, 0), 30000)
    with pytest.raises(b.DsvtError):
        b.dsvt_partition_bound(b.part_cfg((468, 468, 1), (12, 12, 1), (0, 0, 0), 36, 1, 6), 30000)      # inner orders are 0..5
    with pytest.raises(b.DsvtError):
        b.dsvt_partition_bound(b.part_cfg((468, 468, 32), (48, 48, 32), (0, 0, 0), 36, 1, 2), 30000)   # shuffled order: window volume <= 65536


def test_bench_refuses_more_than_one_gpu():
    """bench.py is single-GPU by design: any other --gpus value exits with a message before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_reports_layer_traffic_only_for_the_sources_it_was_measured_with(tmp_path, monkeypatch):
    """bench.py takes the layer kernel's HBM bytes per launch from profiles/k_layer_hbm_traffic.txt, by workload, and
    only when the file's hash of layer.hip + mma.h is that of the sources in the tree."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    f = tmp_path / "traffic.txt"
    f.write_text("# comment\n"
                 f"workload=frame commit=abc1234 sources={bench.layer_source_hash()} fetch_kib=100 write_kib=28\n"
                 "workload=voxel commit=abc1234 sources=0000000000000000 fetch_kib=1 write_kib=1\n")
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    nbytes, where = bench.layer_traffic("frame")
    assert nbytes == 128 * 1024 and "abc1234" in where
    assert bench.layer_traffic("voxel")[0] is None and "other kernel sources" in bench.layer_traffic("voxel")[1]
    assert bench.layer_traffic("skewed") == (None, "not measured for this workload")
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "missing.txt"))
    assert bench.layer_traffic("frame") == (None, "no traffic file")


def test_committed_traffic_file_matches_the_committed_kernel_sources():
    """The tracked traffic figures belong to the tracked layer.hip and mma.h (a change to either needs a new measurement)."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    for w in ("frame", "skewed", "voxel"):
        nbytes, where = bench.layer_traffic(w)
        assert nbytes is not None and nbytes > 0, (w, where)
