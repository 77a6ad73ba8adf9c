"""The host half of the library under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the
library is built once more with the sanitizers on its host code, a C driver sweeps the argument checks,
the workspace sizing (which runs every launch-shape choice of the kernels) and the Eq. 7-8 utilities over
the legal parameter range and its edges, and any finding aborts it.  No kernel runs."""
import os
import subprocess

from paper_2603_14549_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = os.path.join(os.path.dirname(os.path.realpath(build.HIPCC)), "..", "lib", "llvm", "bin", "clang")


def test_host_entry_points_under_asan_and_ubsan(tmp_path):
    out = str(tmp_path)
    lib = build.build_sanitized_host(out)
    clang = CLANG if os.path.exists(CLANG) else "/opt/rocm/lib/llvm/bin/clang"
    exe = os.path.join(out, "host_sweep")
    subprocess.run([clang, "-std=c11", "-D_DEFAULT_SOURCE", "-O1", "-g", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "host_sanitize_driver.c"), lib, "-lm",
                    f"-Wl,-rpath,{out}", "-o", exe], check=True, capture_output=True, text=True)
    env = dict(os.environ)
    # other preloaded libraries may come before the sanitizer runtime in the link order
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    res = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, f"exit {res.returncode}\n{res.stdout[-2000:]}\n{res.stderr[-4000:]}"
    assert "host sweep ok" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
