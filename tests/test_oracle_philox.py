"""Pin of the oracle's Philox4x32-10 against rocRAND's engine (AMD's own,
independent implementation of the Salmon et al. generator), compiled for the
host from the header shipped with ROCm."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import tm_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def _checker(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    exe = str(tmp_path_factory.mktemp("philox") / "philox_rocrand_check")
    subprocess.check_call([hipcc, "-O1", "--offload-arch=gfx950", os.path.join(HERE, "philox_rocrand_check.cpp"),
                           "-o", exe], stderr=subprocess.DEVNULL)
    return exe


def test_philox_matches_rocrand(tmp_path_factory):
    exe = _checker(tmp_path_factory)
    rng = np.random.default_rng(7)
    cases = [(0, 0, 0, 0, 0, 0), (0xffffffff,) * 6]
    for _ in range(400):
        cases.append(tuple(int(v) for v in rng.integers(0, 2**32, size=6, dtype=np.uint64)))
    # counters shaped like the ones the method uses: (blk|stream<<28, g, i, epoch)
    for stream in range(4):
        for blk in (0, 1, 5, 199):
            cases.append((123, 456, blk | (stream << 28), 19999, 59999, 7))
    text = "".join("%x %x %x %x %x %x\n" % c for c in cases)
    out = subprocess.run([exe], input=text, capture_output=True, text=True, check=True).stdout.split("\n")
    for c, line in zip(cases, out):
        want = [int(w, 16) for w in line.split()]
        got = O.philox(list(c[2:]), list(c[:2]))
        assert got == want, (c, got, want)


def test_philox_bits_look_uniform():
    # mean of each output bit over 4096 consecutive counters is near 1/2
    acc = np.zeros(128)
    nblk = 4096
    for b in range(nblk):
        w = O.philox([b, 3, 5, 9], [42, 0])
        bits = np.unpackbits(np.array(w, dtype="<u4").view(np.uint8), bitorder="little")
        acc += bits
    assert np.all(np.abs(acc / nblk - 0.5) < 5 * 0.5 / np.sqrt(nblk))
