"""Host-side sanitizer builds (CPU only): the oracle, and the host half of the library, compiled with
AddressSanitizer and UndefinedBehaviorSanitizer and driven through small C programs (tests/native/) that walk the
validation and refusal paths and a spread of small oracle steps over exact-size heap arrays.  Device code is not
sanitized (the option is given to the host compilation only)."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


@pytest.mark.parametrize("real", ["float", "double"])
def test_oracle_under_asan_and_ubsan(tmp_path, real):
    exe = str(tmp_path / "oracle_san")
    r = run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", f"-DREAL={real}", os.path.join(ROOT, "oracle", "eco_oracle.c"),
             os.path.join(NATIVE, "oracle_san.c"), "-o", exe, "-lm"])
    assert r.returncode == 0, r.stdout
    r = run([exe], env=dict(ENV, OMP_NUM_THREADS="4"), timeout=300)
    assert r.returncode == 0 and r.stdout.strip().startswith("ok"), r.stdout[-3000:]
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout


def test_library_host_code_under_asan_and_ubsan(tmp_path):
    from paper_2601_22101_amd import build
    hipcc = build._hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("hipcc is not available")
    lib = str(tmp_path / "libeco_san.so")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    csrc = os.path.join(ROOT, "paper_2601_22101_amd", "csrc")
    # the host half lives in eco_api.cpp (validation, plans, dispatch) and in the launchers of the kernel files
    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        r = run([hipcc, *build.HIPCC_FLAGS, "-g", *san, "-x", "hip", "-c", os.path.join(csrc, src), "-o", obj])
        assert r.returncode == 0, r.stdout[-3000:]
        return obj
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, build.SOURCES))
    r = run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", *objs, "-o", lib])
    assert r.returncode == 0, r.stdout[-3000:]
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    exe = str(tmp_path / "abi_san")
    r = run([clang, "-O1", "-g", "-std=c99", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-shared-libsan",
             "-I", os.path.join(ROOT, "include"), os.path.join(NATIVE, "abi_san.c"), lib, f"-Wl,-rpath,{tmp_path}", "-o", exe])
    assert r.returncode == 0, r.stdout[-3000:]
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    env = dict(ENV, LD_LIBRARY_PATH=os.pathsep.join([os.path.dirname(rt), "/opt/rocm/lib", os.environ.get("LD_LIBRARY_PATH", "")]))
    r = run([exe], env=env, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-3000:]
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout
