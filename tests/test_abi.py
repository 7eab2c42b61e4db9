"""The shared library loads and exports exactly what include/mgwfbp.h declares (no compute calls)."""
import ctypes
import os
import re
import shutil
import subprocess

import pytest

import paper_1912_09268_amd as M
from paper_1912_09268_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "mgwfbp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mgwfbp_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = _declared()
    for must in ("mgwfbp_plan", "mgwfbp_pack", "mgwfbp_reduce", "mgwfbp_unpack_update", "mgwfbp_group_pipeline",
                 "mgwfbp_ctx_create", "mgwfbp_ctx_destroy", "mgwfbp_eval"):
        assert must in names


def test_library_exports_every_declared_symbol():
    handle = ctypes.CDLL(M.library_path())
    for name in _declared():
        assert hasattr(handle, name), f"{name} declared in mgwfbp.h but not exported"


def test_binding_covers_every_declared_symbol():
    assert sorted(binding._SIGNATURES) == _declared()


def test_version_string_and_error_paths_without_gpu():
    assert M.lib().mgwfbp_version().startswith(b"mgwfbp")
    with pytest.raises(M.MgwfbpError):
        M.Context([4, 4], [0, 1], P=0, host_only=True)            # P out of range
    with pytest.raises(M.MgwfbpError):
        M.Context([4, 4], [1, 0], P=2, host_only=True)            # layer 1 marked merged
    with pytest.raises(M.MgwfbpError):
        M.Context([4, 4], [0, 1], P=2, grad_dtype=7, host_only=True)
    ctx = M.Context([4, 4], [0, 1], P=2, host_only=True)
    with pytest.raises(M.MgwfbpError) as e:                       # device call on a host-only context
        ctx.pack(0, 1, 1)
    assert e.value.status == -1
    ctx.close()


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setenv("MGWFBP_LIBRARY", "/nonexistent/libmgwfbp.so")
    monkeypatch.setattr(binding, "_LIB", None)
    with pytest.raises(M.MgwfbpError):
        M.plan([4], [1.0], 1.0, 1.0)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_plain_c_client_links_and_agrees_with_the_oracle(tmp_path):
    """include/mgwfbp.h compiles as strict C99 and a C program drives plan -> eval -> layout through the
    shared library; its output is compared with the oracle's Algorithm 1, Eq. 8 and Sec. 5.3 layout."""
    import numpy as np
    from oracle import plan as OP
    lib = M.library_path()
    exe = str(tmp_path / "c_abi_client")
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_client.c"), "-o", exe, lib,
           "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    rng = np.random.default_rng(5)
    L = 40
    sizes = [int(4 * x) for x in rng.integers(0, 5000, L)]
    t_b = [float(x) for x in rng.uniform(1e-5, 3e-4, L)]
    a, b = 5e-5, 2e-9
    text = f"{L} {a!r} {b!r}\n" + "".join(f"{s} {t!r}\n" for s, t in zip(sizes, t_b))
    r = subprocess.run([exe], input=text, capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, r.stderr
    out = r.stdout.split("\n")
    merged = OP.plan_algorithm1(sizes, t_b, a, b)
    groups = OP.groups_in_arrival_order(merged)
    assert 0 < sum(merged) < L - 1                               # the instance exercises both branches
    assert out[0] == f"groups {len(groups)}"
    assert float(out[1].split()[1]) == OP.iteration_time(merged, sizes, t_b, a, b)
    assert [int(x.split()[2]) for x in out[2:2 + L]] == merged
    grp, off, sizes_g = OP.merge_layout([s // 4 for s in sizes], merged)
    for i in range(L):
        assert out[2 + L + i] == f"tensor {i} group {grp[i]} off {off[i]}"
    for k in range(len(groups)):
        assert out[2 + 2 * L + k] == f"group {k} elems {sizes_g[k]}"
    assert out[2 + 2 * L + len(groups)] == "device_call_on_host_ctx -1"
    assert out[3 + 2 * L + len(groups)] == "negative_a -1"


def test_product_code_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing in the package or its native sources may import, read or
    mention it, and bench.py may use it only inside its CPU-baseline function."""
    pkg = os.path.join(ROOT, "paper_1912_09268_amd")
    for folder, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                assert "oracle" not in open(os.path.join(folder, f)).read(), f
    assert "oracle" not in open(os.path.join(ROOT, "include", "mgwfbp.h")).read()
    gen = open(os.path.join(ROOT, "workloads.py")).read()          # shared input generators: no imports of either side
    assert "import oracle" not in gen and "from oracle" not in gen and "paper_1912_09268_amd" not in gen
    bench = open(os.path.join(ROOT, "bench.py")).read()
    start = bench.index("def cpu_baseline")
    end = bench.index("\ndef ", start + 1)
    outside = bench[:start] + bench[end:]
    assert "import oracle" not in outside and "from oracle" not in outside
