"""The C-ABI library builds, loads and exports every entry point that include/rh.h declares;
host-only helpers behave (no GPU needed, no compute calls)."""
import ctypes as C
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, n)).read() for n in sorted(os.listdir(inc)) if n.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rh_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2407_16990_amd as pkg
    lib = pkg.load_library()
    names = declared_functions()
    assert {"rh_create", "rh_destroy", "rh_select_regions", "rh_pack", "rh_enhance", "rh_unpack",
            "rh_read_counts", "rh_last_error", "rh_budget", "rh_identity_places", "rh_set_stream",
            "rh_temporal_phi", "rh_temporal_select", "rh_temporal_spread", "rh_select_regions_noalloc"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layouts_match_header_comments():
    import paper_2407_16990_amd as pkg
    assert pkg.BOX_DTYPE.itemsize == 24 and pkg.PLACE_DTYPE.itemsize == 16
    assert C.sizeof(pkg.Config) == 16 * 4 and C.sizeof(pkg.Segment) == 16


def test_budget_host_helper():
    import paper_2407_16990_amd as pkg
    lib = pkg.load_library()
    assert lib.rh_budget(128, 128, 1) == 64 and lib.rh_budget(96, 96, 117) == (96 * 96 * 117) // 256
    assert lib.rh_budget(64, 64, 0) == 0


def test_null_arguments_are_rejected_without_a_gpu():
    import paper_2407_16990_amd as pkg
    lib = pkg.load_library()
    h = C.c_void_p()
    assert lib.rh_create(None, None, 0, None, C.byref(h)) == 1
    cfg = pkg.Config(8, 64, 1, 4, 64, 4, 8, 0, 0, pkg.NetDesc(0, 4, 2, 2))
    w = np.zeros(8, dtype=np.float32)
    assert lib.rh_create(C.byref(cfg), w.ctypes.data_as(C.c_void_p), 8, None, C.byref(h)) == 2   # frame narrower than one macroblock
    assert lib.rh_select_regions(None, None, 1, None, 0, 0, None, None, None) == 1
    assert lib.rh_last_error(None) == b"null context"


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message instead of printing a figure (one-GPU build)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and not r.stdout.strip()


def test_new_entry_points_reject_null_arguments():
    import paper_2407_16990_amd as pkg
    lib = pkg.load_library()
    assert lib.rh_enhance_exact(None, None, 1, None, None, None, None) == 1
    assert lib.rh_enhance_masked(None, None, 1, None, None, None, None) == 1
    assert lib.rh_enhance_needed(None, None, 1, None, None, None, None) == 1
    assert lib.rh_needed_radii(None, 0, None, 0) == -1
    assert lib.rh_temporal_phi(None, None, 1, 0, 1, None) == 1
    assert lib.rh_temporal_select(None, None, None, 1, 1, None, None, None, None) == 1
    assert lib.rh_temporal_spread(None, None, 1, None, None) == 1
    assert lib.rh_select_regions_noalloc(None, 1, 1, 1, None, 0, 0, None, None, None, None) == 1
    assert lib.rh_select_regions_noalloc(None, 5000, 1, 1, None, 0, 0, None, None, None, None) == 3   # beyond the fixed tables
