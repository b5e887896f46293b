"""The library's dynamic-offloading window logic (csrc/lmc_window.hpp, paper section 5.3)
against the oracle's model on random operation sequences, on the CPU, with UBSan."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from oracle.offload_window import OffloadWindowOracle

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("win") / "window_shim.so")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-shared", "-fPIC", "-fsanitize=undefined",
                           "-fno-sanitize-recover=all", "-static-libubsan", "-Wall", "-Wextra",
                           os.path.join(HERE, "native", "window_shim.cpp"), "-o", so])
    lib = ctypes.CDLL(so)
    lib.win_new.restype = ctypes.c_void_p
    lib.win_new.argtypes = [ctypes.c_int64]
    lib.win_delete.argtypes = [ctypes.c_void_p]
    lib.win_release.argtypes = [ctypes.c_void_p, ctypes.c_int64]
    lib.win_take_scheduled.restype = ctypes.c_int64
    lib.win_take_scheduled.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    lib.win_completed.argtypes = [ctypes.c_void_p, ctypes.c_int64]
    lib.win_acquire.restype = ctypes.c_int
    lib.win_acquire.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    lib.win_get.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    return lib


def _get(lib, w):
    out = (ctypes.c_int64 * 5)()
    lib.win_get(w, out)
    return list(out)


@pytest.mark.parametrize("window", [1, 2, 5, 16, 100])
def test_window_logic_matches_oracle(shim, window):
    rng = np.random.default_rng(window)
    ora = OffloadWindowOracle(window)
    w = shim.win_new(window)
    buf = (ctypes.c_int64 * 4096)()
    issued = []            # pages handed to "the store" but not yet complete, in order
    nxt = 0
    for step in range(5000):
        op = rng.integers(0, 4)
        if op == 0:
            for _ in range(rng.integers(1, 6)):
                shim.win_release(w, int(nxt * 3 + 1))
                ora.release(nxt * 3 + 1)
                nxt += 1
        elif op == 1:
            # the store takes some scheduled pages; the oracle's scheduled list is [current, end)
            n = shim.win_take_scheduled(w, int(rng.integers(1, 9)), buf)
            want = ora.scheduled()[len(issued):len(issued) + n]
            assert list(buf[:n]) == want, step
            issued += want
        elif op == 2 and issued:
            n = int(rng.integers(1, len(issued) + 1))
            shim.win_completed(w, n)
            ora.offloaded(n)
            issued = issued[n:]
        elif op == 3:
            n = int(rng.integers(1, 8))
            r = shim.win_acquire(w, n, buf)
            got = ora.take(n)
            if got is None:
                assert r in (1, 2), step
            else:
                assert r == 0 and list(buf[:n]) == got, step
        g = _get(shim, w)
        assert g[:4] == [ora.start, ora.current, ora.end, ora.tail], step
        assert g[4] == ora.state(), step
    shim.win_delete(w)
