"""The host side of the C-ABI library under AddressSanitizer and UndefinedBehaviorSanitizer: an instrumented copy
of the library (host code only; the device code is compiled as usual) is built into a temporary directory and a
small C++ program (tests/abi_sanitizer_driver.cpp) walks every entry point's argument validation against it.
No GPU is needed.  The same build works by hand:
    python -m paper_2404_05567_amd.build -Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined
(that overwrites the in-tree library; load it into Python only with the sanitizer runtime preloaded)."""
import os
import subprocess

from paper_2404_05567_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
       "-Xarch_host", "-fno-omit-frame-pointer"]


def test_abi_argument_validation_is_clean_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "libdsmoe_san.so")
    build.build(verbose=False, extra_flags=SAN, lib_path=lib, obj_dir=str(tmp_path),
                link_flags=["-fsanitize=address", "-fsanitize=undefined"])
    exe = str(tmp_path / "abi_driver")
    subprocess.check_call([build.HIPCC, "-x", "c++", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined",
                           "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "abi_sanitizer_driver.cpp"), "-x", "none", lib,
                           f"-Wl,-rpath,{tmp_path}", "-o", exe])
    env = dict(os.environ)
    # other preloaded libraries may come first in the link order; leak checks would also see the HIP runtime's own
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    p = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 0, p.stdout
    assert "all checks passed" in p.stdout, p.stdout
    assert "AddressSanitizer" not in p.stdout and "runtime error" not in p.stdout, p.stdout
