"""Host code under sanitizers (no GPU).  (1) The C oracle under AddressSanitizer and
UndefinedBehaviorSanitizer: a small driver calls every entry on seeded cases with exactly sized heap
buffers, including empty active sets, k larger than a set, an empty batch union, clusters that lose their
members, recorded tokens outside the vocabulary and missing beam candidates.  (2) The host side of the C
ABI under AddressSanitizer: every argument check that runs before any GPU work."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = ["vp_oracle.c", "vp_train_oracle.c", "vp_search_oracle.c"]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitize"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", os.path.join(ROOT, "tests", "oracle_sanitize_main.c")]
    cmd += [os.path.join(ROOT, "oracle", s) for s in SOURCES] + ["-lm", "-o", str(exe)]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitizer run ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr


HIPCC = "/opt/rocm/bin/hipcc"
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
API_SOURCES = ["vp_api.hip", "train_api.hip", "search.hip"]   # every file that defines a function of include/vp.h


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="needs hipcc and its clang++")
def test_host_side_of_the_c_abi_runs_clean_under_address_sanitizer(tmp_path):
    """The files that define the C ABI rebuilt with the host pass under AddressSanitizer (device code as
    always), linked over the in-tree library for the kernel launchers, and driven through every check that
    happens before any GPU work.  No GPU needed."""
    from paper_2208_06874_amd import vp
    if not os.path.exists(vp.LIB_PATH):
        pytest.skip("libvp.so is not built")
    csrc = os.path.join(ROOT, "paper_2208_06874_amd", "csrc")
    inc = os.path.join(ROOT, "include")
    objs = []
    for src in API_SOURCES:
        obj = tmp_path / (src + ".o")
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC",
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-Xarch_host", "-fsanitize=address", "-I", inc, "-I", csrc,
                        "-c", os.path.join(csrc, src), "-o", str(obj)], check=True, capture_output=True)
        objs.append(str(obj))
    # the driver is plain C++ (hipcc would take every input of a line with a .cpp for HIP source)
    main_o = tmp_path / "main.o"
    subprocess.run([CLANGXX, "-O1", "-g", "-std=c++17", "-fsanitize=address", "-I", inc, "-c",
                    os.path.join(ROOT, "tests", "boundary_sanitize_main.cpp"), "-o", str(main_o)],
                   check=True, capture_output=True)
    exe = tmp_path / "boundary_sanitize"
    libdir = os.path.dirname(vp.LIB_PATH)
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fno-gpu-sanitize", str(main_o), *objs,
                    "-L", libdir, "-lvp", "-Wl,-rpath," + libdir, "-o", str(exe)], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "boundary sanitizer run ok" in r.stdout
    assert "AddressSanitizer" not in r.stderr, r.stderr
