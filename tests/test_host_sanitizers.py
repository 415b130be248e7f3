"""The host builder under AddressSanitizer and UBSan (host code only), with range checks on
every emitted work item, stream entry and scratch slot."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_builder_is_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2409_02208_amd", "csrc"), os.path.join(ROOT, "tests", "host_sanitize_main.cpp"),
           os.path.join(ROOT, "paper_2409_02208_amd", "csrc", "cbm_builder.cpp"), "-o", exe, "-lpthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "sanitize" in r.stderr:
        pytest.skip("sanitizer runtime not available: " + r.stderr[-200:])
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "asan run ok" in r.stdout, (r.stdout[-500:], r.stderr[-3000:])
    # once more with every multi-row round emitted as bundles (one sweep per path, rows tagged in the entries)
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(env, CBM_BUNDLE_MIN="1", CBM_BUNDLE_MIN_ITEMS="1"), timeout=300)
    assert r.returncode == 0 and "asan run ok" in r.stdout, (r.stdout[-500:], r.stderr[-3000:])


def test_header_is_valid_c():
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "cbm.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
