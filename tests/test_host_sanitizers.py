"""The library's host-side scene builder (plain C++, no device call) under AddressSanitizer +
UndefinedBehaviorSanitizer: valid scenes of every kind and size class, and descriptions it must reject."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_scene_builder_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "scene_sanitize")
    csrc = os.path.join(ROOT, "paper_2502_00021_amd", "csrc")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                           "-I", os.path.join(ROOT, "include"), "-I", csrc,
                           os.path.join(csrc, "scene.cpp"), os.path.join(ROOT, "tests", "scene_sanitize_main.cpp"),
                           "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    sys.stdout.write(r.stdout)
    sys.stderr.write(r.stderr[-4000:])
    assert r.returncode == 0, r.stderr[-2000:]
    assert r.stdout.startswith("ok ")
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
