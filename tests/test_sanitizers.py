"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code, on the CPU only.

Two instrumented builds are made in a temporary folder: the oracle (all of it is host
code) and the C ABI's host translation unit, ``csrc/api.cpp`` (argument checks, sizes,
dispatch, Cook-Toom construction), linked with the ordinary objects of the kernels.
The oracle pins and the boundary tests then run again in a child interpreter that has
the sanitizer runtime preloaded; any report ends the child with a non-zero status.
Device code is not instrumented: GPU sanitizer runs are not available on the target
machines, and nothing here touches a GPU.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2002_10711_amd")
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
       "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]


def _gcc_file(name):
    out = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True,
                         text=True, check=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


LIBASAN = _gcc_file("libasan.so") if shutil.which("gcc") else None
pytestmark = pytest.mark.skipif(LIBASAN is None, reason="gcc's libasan.so is not installed")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-4000:], r.stderr[-4000:])
    return r


def _child_env(extra):
    env = dict(os.environ)
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = LIBASAN + (":" + pre if pre else "")
    # The interpreter itself is not instrumented, so its deliberate leaks say nothing.
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SANITIZED_CHILD"] = "1"
    env.update(extra)
    return env


def _pytest_child(files, env):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + files
    r = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT, env=env)
    text = r.stdout + r.stderr
    assert "runtime error" not in text and "AddressSanitizer" not in text, text[-6000:]
    assert r.returncode == 0, text[-6000:]
    assert " passed" in text
    return text


@pytest.fixture(scope="module")
def san_dir(tmp_path_factory):
    return str(tmp_path_factory.mktemp("san"))


def test_oracle_under_asan_ubsan(san_dir):
    so = os.path.join(san_dir, "liboracle_san.so")
    _run(["g++"] + SAN + ["-fopenmp", "-shared", "-fPIC", "-o", so,
                          os.path.join(ROOT, "oracle", "wino_oracle.cpp")])
    _pytest_child(["tests/test_oracle_pins.py"], _child_env({"WINO_ORACLE_LIB": so}))


def test_c_abi_host_code_under_asan_ubsan(san_dir):
    from paper_2002_10711_amd import build as wb

    objdir = wb.OBJ
    want = [os.path.join(objdir, os.path.basename(s) + ".o") for s in wb.sources()]
    if not all(os.path.exists(o) for o in want):
        wb.build()
    api_o = os.path.join(san_dir, "api_san.o")
    # api.cpp holds no device code: g++ compiles it as plain C++ against the HIP headers.
    _run(["g++", "-x", "c++", "-std=c++17"] + SAN +
         ["-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
          "-I" + wb.CSRC, "-fPIC", "-c", os.path.join(wb.CSRC, "api.cpp"), "-o", api_o])
    so = os.path.join(san_dir, "libwino_san.so")
    objs = [o for o in want if not o.endswith("api.cpp.o")]
    _run([wb.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", so, api_o] + objs +
         ["-L" + os.path.dirname(LIBASAN), "-lasan", "-lubsan"])
    _pytest_child(["tests/test_boundary.py"], _child_env({"WINO_LIB": so}))
