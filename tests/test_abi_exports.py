"""The C-ABI library loads and exports every function that include/mobile_moe.h declares; host-side
argument validation returns the documented codes without touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2510_12357_amd import binding as mm
from paper_2510_12357_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mobile_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?[A-Za-z_][\w\s\*]*?\b(\w+)\s*\([^;{]*\)\s*;", text, flags=re.M)
    return sorted(set(names))


def test_header_functions_are_exported():
    if not os.path.exists(mm.LIB_PATH):
        pytest.skip("libmobile_moe.so not built (python -m paper_2510_12357_amd.build)")
    lib = ctypes.CDLL(mm.LIB_PATH)
    names = declared_functions()
    assert len(names) >= 15 and "moe_route" in names and "expert_cache_fetch" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mobile_moe.h but not exported"
    assert set(mm.EXPORTS) == set(names)


def test_config_validation_codes_without_gpu():
    if not os.path.exists(mm.LIB_PATH):
        pytest.skip("libmobile_moe.so not built")
    base = wl.CONFIGS["fine60_decode"]
    assert mm.moe_dispatch_workspace_bytes(mm.make_config(base)) >= 4 * base.E
    need = mm.moe_expert_ffn_workspace_bytes(mm.make_config(base))
    assert need >= 2 * (base.T * base.k_big * base.I + base.T * base.shared_I[0])
    lib = mm.load_library()
    for bad, code in ((base.with_(k_little=5), -2), (base.with_(H=2052), -3), (base.with_(E=300), -3),
                      (base.with_(k_big=70, k_little=1, E=80), -3), (base.with_(T=-1), -2)):
        c = mm.make_config(bad)
        assert mm.moe_dispatch_workspace_bytes(c) == 0
        rc = lib.moe_combine(ctypes.byref(c), None, None, None, None, None, None, None)
        assert rc == code, (bad, rc, mm.moe_last_error())
        assert mm.moe_last_error()


def test_bench_refuses_more_than_one_gpu():
    """Every box of this build has one GPU: the benchmark says so instead of starting ranks."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "single-GPU" in (r.stderr + r.stdout)
