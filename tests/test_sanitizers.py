"""CPU-only sanitizer leg: the oracle's C entry points and every argument-error path of the C ABI run under
AddressSanitizer and UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU)."""
import os
import shutil
import subprocess

import pytest

import paper_2411_02886_amd as ts

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=77", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


@pytest.fixture(scope="module")
def gcc(tmp_path_factory):
    cc = shutil.which("gcc")
    if cc is None:
        pytest.skip("no C compiler")
    d = tmp_path_factory.mktemp("san")
    probe = d / "probe.c"
    probe.write_text("int main(void) { return 0; }\n")
    r = subprocess.run([cc, *SAN, str(probe), "-o", str(d / "probe")], capture_output=True, text=True)
    if r.returncode != 0 or subprocess.run([str(d / "probe")], env=ENV).returncode != 0:
        pytest.skip("this gcc cannot build or run sanitized programs")
    return cc, d


def test_oracle_entry_points_under_asan_and_ubsan(gcc):
    cc, d = gcc
    exe = str(d / "oracle_sanitizer_driver")
    subprocess.check_call([cc, "-std=c99", "-Wall", *SAN, os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"), "-o", exe, "-lm"])
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"].replace("detect_leaks=0", "detect_leaks=1")))
    assert r.returncode == 0 and "ran clean" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])


def test_every_abi_error_path_under_asan_and_ubsan(gcc):
    # the program is instrumented; libtokenselect.so (HIP host code) is not, but every call returns from its argument
    # checks.  Leak checking is off: the HIP runtime the library pulls in keeps process-lifetime allocations.
    cc, d = gcc
    libdir = os.path.dirname(ts.lib_path())
    exe = str(d / "c_abi_check_san")
    subprocess.check_call([cc, "-std=c99", "-Wall", "-Wextra", *SAN, "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", exe, "-L", libdir, "-ltokenselect",
                           "-Wl,-rpath," + libdir])
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV)
    assert r.returncode == 0 and "c abi ok" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
