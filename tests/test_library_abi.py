"""The built C-ABI library loads and exports every function the header declares (CPU only;
no compute call is made)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "infaas_sel.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(infaas_sel_[a-z_]+)\s*\(", text)))


def test_header_declares_the_five_calls():
    names = _declared()
    for n in ("infaas_sel_create", "infaas_sel_load_variants", "infaas_sel_update_load",
              "infaas_sel_select", "infaas_sel_destroy"):
        assert n in names


def test_library_exports_every_declared_symbol():
    import paper_1905_13348_amd as pkg
    from paper_1905_13348_amd.binding import EXPORTED
    if not os.path.exists(pkg.library_path()):
        pytest.skip("library not built here (run __graft_entry__.build())")
    lib = pkg.load_library()
    declared = _declared()
    assert sorted(EXPORTED) == declared
    for n in declared:
        assert hasattr(lib, n), n


def test_status_text():
    import paper_1905_13348_amd as pkg
    if not os.path.exists(pkg.library_path()):
        pytest.skip("library not built here")
    lib = pkg.load_library()
    assert lib.infaas_sel_strerror(0) == b"ok"
    assert lib.infaas_sel_strerror(-2) == b"no variant table loaded"
    # null handles are rejected without touching a device
    assert lib.infaas_sel_select(None, 1, None, None, None, None, None, None) == -1
    assert lib.infaas_sel_update_load(None, 1, None, None, None) == -1
    lib.infaas_sel_destroy(None)


def test_create_rejects_bad_configs_before_touching_a_device():
    """Argument checks of infaas_sel_create come before any HIP call, so they work without a GPU."""
    import ctypes
    import paper_1905_13348_amd as pkg
    from paper_1905_13348_amd.binding import _Config
    if not os.path.exists(pkg.library_path()):
        pytest.skip("library not built here")
    lib = pkg.load_library()
    h = ctypes.c_void_p()
    assert lib.infaas_sel_create(None, ctypes.byref(h)) == -1
    for kw in (dict(num_tasks=0, num_batch_sizes=1), dict(num_tasks=1, num_batch_sizes=0),
               dict(num_tasks=1, num_batch_sizes=65), dict(num_tasks=1 << 22, num_batch_sizes=8),
               dict(num_tasks=1, num_batch_sizes=1, flags=7), dict(num_tasks=1, num_batch_sizes=1, flags=16),
               dict(num_tasks=1, num_batch_sizes=1, lds_segment_limit=63),
               dict(num_tasks=1, num_batch_sizes=1, lds_segment_limit=9000)):
        cfg = _Config(batch_sizes=None, device=0, **kw)
        assert lib.infaas_sel_create(ctypes.byref(cfg), ctypes.byref(h)) == -1, kw
        assert not h.value
    assert lib.infaas_sel_load_variants(None, 0, None, None, None, None, None) == -1
    assert lib.infaas_sel_reserve(None, 10) == -1
    assert lib.infaas_sel_get_info(None, None) == -1


def test_product_does_not_touch_the_oracle():
    """The package and the C/HIP sources never import, include or name the oracle."""
    pkg_dir = os.path.join(ROOT, "paper_1905_13348_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
    assert "oracle" not in open(os.path.join(ROOT, "include", "infaas_sel.h")).read().lower()


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N above 1 exits with a message and touches no GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
