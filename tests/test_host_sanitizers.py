"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer, no GPU needed: the CPU oracle's
C source and the host side of the library's C ABI (argument checks and the search planner, swept
over a grid of shapes through lpq_search_plan_info) are compiled with the sanitizers (host pass
only: the device code is built as always) and driven by tests/host/san_driver.cpp."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG_DIR = "/opt/rocm/lib/llvm/bin"
SAN = "address,undefined"


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    return r


@pytest.fixture(scope="module")
def built(tmp_path_factory):
    from paper_2110_08919_amd import build as lib_build
    if not os.path.exists(os.path.join(CLANG_DIR, "clang++")):
        pytest.skip("no clang next to hipcc")
    lib_build.build()                                      # the ordinary objects (device code, other translation units)
    out = str(tmp_path_factory.mktemp("san"))
    # host side of the C ABI and the planner, instrumented on the host pass only
    api_o = os.path.join(out, "api.san.o")
    _run([lib_build.HIPCC, *lib_build.FLAGS, "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
          "-Xarch_host", "-fno-sanitize-recover=all", "-c", os.path.join(lib_build.CSRC, "api.hip"), "-o", api_o])
    others = [os.path.join(lib_build.OBJ, os.path.basename(s)[:-4] + ".o") for s in lib_build.sources()
              if not s.endswith("api.hip")]
    lib = os.path.join(out, "liblpq_san.so")
    _run([lib_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, api_o, *others])
    # the oracle (plain C, no OpenMP here) and the driver, same sanitizers, same compiler family
    oracle_o = os.path.join(out, "oracle.san.o")
    _run([os.path.join(CLANG_DIR, "clang"), "-O1", "-g", "-std=c11", "-ffp-contract=off", f"-fsanitize={SAN}",
          "-fno-sanitize-recover=all", "-c", os.path.join(ROOT, "oracle", "lpq_oracle.c"), "-o", oracle_o])
    exe = os.path.join(out, "san_driver")
    _run([os.path.join(CLANG_DIR, "clang++"), "-O1", "-g", "-std=c++17", f"-fsanitize={SAN}", "-fno-sanitize-recover=all",
          "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host", "san_driver.cpp"), oracle_o, "-ldl", "-lm", "-o", exe])
    return exe, lib


def test_oracle_planner_and_abi_under_sanitizers(built):
    exe, lib = built
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, lib], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:] + "\n" + r.stderr[-4000:]
    assert "all host checks passed" in r.stdout
    assert "planner:" in r.stdout and "oracle:" in r.stdout
