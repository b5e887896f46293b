"""ThreadSanitizer over the library's host side (context, index, pool bookkeeping): the
host code of liblmc is rebuilt with -fsanitize=thread and six threads hammer one
index-only context through the C ABI, with counted readers and the directory tier's
writer threads reading the pool meanwhile.  CPU only; no HIP call is made."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2510_09665_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="needs hipcc to rebuild the host code")
def test_host_side_is_race_free_under_tsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    lib = str(tmp_path / "liblmc_tsan.so")
    from paper_2510_09665_amd.build import SOURCES       # every source of the library, as the build lists them
    srcs = [os.path.join(CSRC, f) for f in SOURCES]
    build = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
             "-Xarch_host", "-fsanitize=thread", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    res = subprocess.run(build + srcs + ["-o", lib], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    exe = str(tmp_path / "tsan_driver")
    # the driver is plain host C++; the clang that ships with ROCm provides the runtime
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    res = subprocess.run([clang, "-std=c++17", "-O1", "-g", "-fsanitize=thread",
                          os.path.join(HERE, "native", "tsan_driver.cpp"), lib, "-Wl,-rpath," + str(tmp_path),
                          "-Wl,-rpath,/opt/rocm/lib", "-lpthread", "-o", exe],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ)
    env["TSAN_OPTIONS"] = "halt_on_error=1:report_signal_unsafe=0"
    dirs = [str(tmp_path / "tier_a"), str(tmp_path / "tier_b")]
    for d in dirs:
        os.mkdir(d)
    res = subprocess.run([exe] + dirs, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    sys.stdout.write(res.stdout[-3000:])
    assert res.returncode == 0 and res.stdout.strip().endswith("ok"), res.stdout[-3000:]
