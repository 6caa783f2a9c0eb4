"""CPU checks of the library's noise arithmetic (host build of the kernels' own header)
against the oracle: Philox word for word, Box-Muller within a few fp32 ulp."""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

from oracle import flashdp_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def shim():
    d = tempfile.mkdtemp(prefix="flashdp_shim_")
    so = os.path.join(d, "shim.so")
    subprocess.check_call(["g++", "-O2", "-mfma", "-ffp-contract=fast", "-shared", "-fPIC", "-o", so,
                           os.path.join(HERE, "host_math_shim.cpp")])
    return ctypes.CDLL(so)


def _u32p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))


def test_library_philox_matches_known_answers(shim, golden_dir):
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        rows = [[int(x, 16) for x in l.split()] for l in f if l.strip() and not l.startswith("#")]
    for w in rows:
        ctr = np.array(w[0:4], np.uint32)
        key = np.array(w[4:6], np.uint32)
        out = np.zeros(4, np.uint32)
        shim.shim_philox(_u32p(ctr), _u32p(key), _u32p(out))
        assert out.tolist() == w[6:10]


def test_library_box_muller_close_to_oracle(shim):
    rng = np.random.default_rng(7)
    words = rng.integers(0, 1 << 32, size=(1 << 20, 4), dtype=np.uint64).astype(np.uint32)
    # edge words: smallest / largest uniforms, quadrant boundaries, u just below and above 1/2 and 3/4
    edge = [0, 255, 256, 0xFFFFFFFF, 0xFFFFFF00, 0x80000000, 0x7FFFFFFF, 0x40000000, 0x3FFFFFFF, 0xC0000000,
            0xBFFFFFFF, 0x20000000, 0xE0000000, 0x00000100, 0x00000200, 0x5FFFFFFF, 0x60000000, 0x2FFFFFFF, 0x30000000]
    e = np.array([(a, b, b, a) for a in edge for b in edge], dtype=np.uint32)
    words = np.concatenate([e, words])
    z = np.zeros(words.shape, np.float32)
    shim.shim_box_muller(_u32p(words), ctypes.c_long(words.shape[0]), z.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    want = O.gaussians_from_words(words)
    err = np.abs(z.astype(np.float64) - want)
    assert err.max() < 1.5e-6, err.max()
    assert np.sqrt(np.mean(err ** 2)) < 1.5e-7
    # relative accuracy where the value is not tiny
    big = np.abs(want) > 1e-3
    assert np.max(err[big] / np.abs(want[big])) < 2e-6


def test_library_noise_field_keying(shim):
    seed, layer, n = (9 << 32) | 4, 6, 10007
    z = np.zeros(n, np.float32)
    shim.shim_noise_field(ctypes.c_uint64(seed), ctypes.c_uint32(layer), ctypes.c_long(n),
                          z.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    want = O.noise_field(seed, layer, n)
    assert np.max(np.abs(z - want)) < 1.5e-6
