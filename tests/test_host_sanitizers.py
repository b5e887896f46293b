"""The library's host-side index / allocator / hashing code (csrc/lmc_index.hpp) under
AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU: a native driver runs random
operation sequences against std::map / std::set models."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def test_index_allocator_hash_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "index_sanitize")
    src = os.path.join(HERE, "native", "index_sanitize.cpp")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
                           "-Wall", "-Wextra", src, "-o", exe])
    env = dict(os.environ)
    # the runtime is linked statically, so it need not be first in the library list
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         env=env, timeout=300)
    sys.stdout.write(res.stdout[-2000:])
    assert res.returncode == 0 and res.stdout.strip().endswith("ok"), res.stdout[-2000:]
