"""The host runtime under AddressSanitizer + UBSan (host code only): a C++ driver
replays random pool / hotness / load sequences on dry_run contexts."""
import os
import shutil
import subprocess

import pytest

from paper_2510_20878_amd.build import SOURCES       # every source of the library

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs hipcc")
def test_host_runtime_fuzz_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "fuzz_host")
    csrc = os.path.join(ROOT, "paper_2510_20878_amd", "csrc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           os.path.join(ROOT, "tests", "host_sanitize", "fuzz_host.cpp"),
           *[os.path.join(csrc, f) for f in SOURCES],
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe, "150"], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "fuzz_host ok" in r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs hipcc")
def test_host_runtime_from_four_threads_under_tsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "threads_host")
    csrc = os.path.join(ROOT, "paper_2510_20878_amd", "csrc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=thread", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           os.path.join(ROOT, "tests", "host_sanitize", "threads_host.cpp"),
           *[os.path.join(csrc, f) for f in SOURCES],
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1:exitcode=66")
    r = subprocess.run([exe, "2000"], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "threads_host ok" in r.stdout
    # the same four threads over real files and real bytes: the loads release the context's lock
    # while the I/O threads move the chunks
    pools = tmp_path / "pools"
    pools.mkdir()
    r = subprocess.run([exe, "120", str(pools)], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "threads_host ok" in r.stdout and "O_DIRECT" in r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs hipcc")
def test_pageable_and_file_tiers_with_real_files_under_asan_ubsan(tmp_path):
    """dry_run = 2 contexts: no HIP call, but real host copies and real (also O_DIRECT) files.
    Covers the direct-I/O buffer that a later, larger file slab must not overrun."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "tiers_host")
    csrc = os.path.join(ROOT, "paper_2510_20878_amd", "csrc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           os.path.join(ROOT, "tests", "host_sanitize", "tiers_host.cpp"),
           *[os.path.join(csrc, f) for f in SOURCES],
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    pools = tmp_path / "pools"
    pools.mkdir()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe, str(pools)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "tiers_host ok" in r.stdout
