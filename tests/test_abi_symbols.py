"""The C-ABI library loads without a GPU and exports every entry point the
header declares; the host-only calls work.  CPU only (no compute calls)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import ff_oracle as O
from paper_2602_00397_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


HEADERS = ("fastforward.h", "fastforward_diag.h")


def _declared():
    names = set()
    for h in HEADERS:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(ff_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = _declared()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/*.h but not exported"
    assert sorted(B.EXPORTS) == names          # the binding covers the whole header


def test_struct_layouts_match_header():
    assert ctypes.sizeof(B.Shape) == 24
    assert ctypes.sizeof(B.Predictor) == 24 and ctypes.sizeof(B.FfnWeights) == 24
    assert ctypes.sizeof(B.Compensator) == 24


def test_host_only_calls():
    for d_ffn, s in ((688, 0.5), (14336, 0.25), (14336, 0.75), (18944, 0.5), (7, 0.5), (10, 1.0), (10, 0.0)):
        assert B.k_from_sparsity(d_ffn, s) == O.k_from_sparsity(d_ffn, s)
    with pytest.raises(B.FFError):
        B.k_from_sparsity(10, 1.5)
    g = np.random.default_rng(0)
    for _ in range(20):
        imp = g.random(int(g.integers(2, 40))) + 0.01
        bud = float(g.uniform(0.2, 0.9))
        np.testing.assert_allclose(B.layer_budgets(imp, bud), O.layerwise_budgets(imp, bud), rtol=1e-13)
    with pytest.raises(B.FFError):
        B.layer_budgets([1.0, -1.0], 0.5)
    shp = B.Shape(4096, 14336, 8192, 128, 128, 64)
    need = B.workspace_bytes(shp, 7168)
    assert need >= 8192 * (7168 + 64) * 2             # at least the activations H
    with pytest.raises(B.FFError):
        B.workspace_bytes(B.Shape(100, 14336, 8192, 128, 128, 64), 7168)   # d_model not a multiple of 128
    assert B.load_library().ff_status_str(2) == b"unsupported shape"


def test_library_depends_on_the_hip_runtime_only():
    """The boundary is plain C: the shared library needs the HIP runtime and the C/C++ runtimes,
    nothing of PyTorch or Python."""
    import subprocess
    B.load_library()
    lib_path = os.path.join(ROOT, "paper_2602_00397_amd", "libfastforward.so")
    out = subprocess.run(["readelf", "-d", lib_path], stdout=subprocess.PIPE, text=True, check=True).stdout
    needed = re.findall(r"\(NEEDED\)\s+Shared library: \[([^\]]+)\]", out)
    assert any(n.startswith("libamdhip64") for n in needed)
    for n in needed:
        assert re.match(r"lib(amdhip64|stdc\+\+|m|gcc_s|c|pthread|dl|rt)\.so", n), f"unexpected dependency {n}"


def test_header_is_plain_c(tmp_path):
    """Each header under include/ compiles as C99 on its own (no C++ and no HIP types in the boundary)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    for h in HEADERS:
        src = tmp_path / (h.replace(".", "_") + ".c")
        src.write_text(f'#include "{h}"\nint main(void) {{ ff_shape s; (void)s; return 0; }}\n')
        r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I" + os.path.join(ROOT, "include"),
                            "-fsyntax-only", str(src)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout


def _run_host_checks():
    import subprocess
    exe = os.path.join(ROOT, "paper_2602_00397_amd", "_build", "ff_host_checks")
    if not os.path.exists(exe):
        pytest.skip("ff_host_checks not built (python -c 'import __graft_entry__ as g; g.build()')")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    print(r.stdout)
    assert r.returncode == 0, r.stdout
    assert "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout
    return r.stdout


def test_host_code_under_sanitizers_without_a_gpu():
    """csrc/ff_host_checks.c linked with the library, host code built with AddressSanitizer and
    UndefinedBehaviorSanitizer: the pure host helpers at their edges, every entry point with a NULL
    context, ff_create on devices that do not exist.  (With a GPU present the program goes on to the
    argument errors of every compute call and to real calls: the GPU test below.)"""
    out = _run_host_checks()
    assert "0 wrong" in out


@pytest.mark.gpu
def test_host_code_under_sanitizers_with_a_gpu():
    """The same program on a machine with a GPU: every argument error of every compute call (nothing
    may be launched), then real calls on a tiny layer with unequal K often enough to wrap the staging
    ring, stage timing and list validation on - all host code of the library under the sanitizers."""
    out = _run_host_checks()
    assert "host checks with a GPU" in out and "0 wrong" in out
