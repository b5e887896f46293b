"""The copy-engine guard (csrc/lmc_guard.hpp): host logic that watches the rate of the
runtime's large device-to-host copies and hands them to the library's copy kernel for a
while when they turn slow.  Scenarios written out by hand, on the CPU, with UBSan."""
import ctypes
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
MiB = 1 << 20


@pytest.fixture(scope="module")
def lib(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("guard") / "guard_shim.so")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-shared", "-fPIC", "-fsanitize=undefined",
                           "-fno-sanitize-recover=all", "-static-libubsan", "-Wall", "-Wextra",
                           os.path.join(HERE, "native", "guard_shim.cpp"), "-o", so])
    lib = ctypes.CDLL(so)
    lib.guard_new.restype = ctypes.c_void_p
    lib.guard_free.argtypes = [ctypes.c_void_p]
    lib.guard_observe.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_double, ctypes.c_double]
    lib.guard_use_kernel.argtypes = [ctypes.c_void_p, ctypes.c_double]
    lib.guard_use_kernel.restype = ctypes.c_int
    lib.guard_best.argtypes = [ctypes.c_void_p]
    lib.guard_best.restype = ctypes.c_double
    lib.guard_switches.argtypes = [ctypes.c_void_p]
    lib.guard_switches.restype = ctypes.c_uint64
    return lib


class Guard:
    def __init__(self, lib):
        self.lib, self.g = lib, lib.guard_new()

    def copy(self, gbps, now, nbytes=480 * MiB):
        self.lib.guard_observe(self.g, nbytes, nbytes / (gbps * 1e9), now)

    def kernel(self, now):
        return bool(self.lib.guard_use_kernel(self.g, now))

    def close(self):
        self.lib.guard_free(self.g)


def test_healthy_copies_never_switch(lib):
    g = Guard(lib)
    assert not g.kernel(0.0)
    for i in range(100):
        g.copy(56.0 + (i % 5) * 0.2, 0.01 * i)       # ordinary jitter
        assert not g.kernel(0.01 * i)
    assert lib.guard_switches(g.g) == 0 and 56e9 < lib.guard_best(g.g) < 57e9
    g.close()


def test_two_slow_copies_of_the_last_four_switch_then_the_runtime_is_tried_again(lib):
    g = Guard(lib)
    g.copy(57.0, 0.00)
    g.copy(31.5, 0.01)                                # one slow copy alone is not enough
    assert not g.kernel(0.011)
    for i in range(3):
        g.copy(56.5, 0.02 + 0.001 * i)                # ... and three healthy ones push it out
    g.copy(31.5, 0.03)
    assert not g.kernel(0.031)
    g.copy(56.0, 0.035)                               # the fast small copy at the head of a store
    g.copy(31.5, 0.04)                                # second slow one of the last four: kernel for 0.25 s
    assert g.kernel(0.041) and g.kernel(0.289) and not g.kernel(0.291)
    # the runtime is tried again and is still slow: two probes, then 0.5 s, then 1, 2, 2
    t = 0.3
    for hold in (0.5, 1.0, 2.0, 2.0):
        g.copy(31.5, t)
        assert not g.kernel(t + 0.001)
        g.copy(31.5, t + 0.02)
        assert g.kernel(t + 0.021) and g.kernel(t + 0.02 + hold - 0.001) and not g.kernel(t + 0.02 + hold + 0.001)
        t += 0.02 + hold + 0.01
    # healthy again for a while: back to the runtime, and the next episode starts at 0.25 s again
    for i in range(4):
        g.copy(56.8, t + 0.01 * i)
        assert not g.kernel(t + 0.01 * i + 0.001)
    g.copy(30.0, t + 0.1)
    g.copy(30.0, t + 0.2)
    assert g.kernel(t + 0.44) and not g.kernel(t + 0.46)
    assert lib.guard_switches(g.g) == 6
    g.close()


def test_small_copies_and_a_slow_start_are_ignored(lib):
    g = Guard(lib)
    for i in range(10):                               # 1 MiB copies are bound by latency: no evidence
        g.copy(20.0, 0.001 * i, nbytes=1 * MiB)
    assert lib.guard_best(g.g) == 0.0 and not g.kernel(0.02)
    # a context that starts in the slow state has nothing to compare with ...
    g.copy(31.5, 0.1)
    g.copy(31.5, 0.2)
    assert not g.kernel(0.21)
    # ... until a healthy copy shows what the link can do
    g.copy(56.9, 0.3)
    g.copy(31.5, 0.4)
    g.copy(31.5, 0.5)
    assert g.kernel(0.51)
    # 60 % of the best is the line: 35 GB/s is still fine (a copy that shares the link), 34 is not
    g2 = Guard(lib)
    g2.copy(57.0, 0.0)
    g2.copy(35.0, 0.1)
    g2.copy(35.0, 0.2)
    assert not g2.kernel(0.21)
    g2.copy(34.0, 0.3)
    g2.copy(34.0, 0.4)
    assert g2.kernel(0.41)
    g.close()
    g2.close()
