"""The GPU library's packed-byte trim, built for the host, against the oracle (CPU only)."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))

MODES = [(4, m) for m in (0x1F, 0x15, 0x11, 0x13, 0x17, 0x19, 0x1B, 0x1D)] + \
        [(3, 0x3F), (2, 0x7F), (3, 0x29), (2, 0x55), (3, 0x2B), (3, 0x2D), (2, 0x5F)]


@pytest.fixture(scope="module")
def swar(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("swar") / "libswar_host.so")
    subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-o", so,
                    os.path.join(HERE, "swar_host_check.cpp")], check=True)
    lib = ctypes.CDLL(so)
    lib.swar_all_pairs.argtypes = [ctypes.c_int, ctypes.c_uint, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    return lib


@pytest.mark.parametrize("n,mask", MODES)
@pytest.mark.parametrize("rnd", [0, 1])
@pytest.mark.parametrize("pairing", [0, 1])
def test_packed_trim_equals_oracle_on_all_pairs(oracle, swar, n, mask, rnd, pairing):
    if oracle.mode_check(n, mask, rnd, pairing):
        pytest.skip("mode not valid with pairing")
    out = np.empty((256, 256, 4), dtype=np.uint8)
    swar.swar_all_pairs(n, mask, rnd, pairing, out.ctypes.data_as(ctypes.c_void_p))
    a, b = np.meshgrid(np.arange(256, dtype=np.uint8), np.arange(256, dtype=np.uint8), indexing="ij")
    x = np.stack([a, b, b, a], axis=-1).reshape(-1, 4)
    exp = oracle.trim(x, n, mask, rnd, pairing).reshape(256, 256, 4)
    assert np.array_equal(out, exp)
