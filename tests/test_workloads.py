"""The seeded input generators: same bytes every time (CRCs recorded when the generators were
written), the stated shapes and distributions."""
import zlib

import numpy as np

from paper_2405_02086_amd import workloads

CRC32 = {"small_256x128": "8bca8e8b", "square_4096": "7b5e2741", "paper_1000x10000": "3b4e277f"}


def test_generators_are_reproducible_bit_for_bit():
    for name, crc in CRC32.items():
        w, Y = workloads.make(name)
        assert Y.dtype == np.float32 and Y.flags["C_CONTIGUOUS"] and Y.shape == tuple(w.shape)
        assert "%08x" % zlib.crc32(Y.tobytes()) == crc, name
        assert np.array_equal(workloads.make(name)[1], Y)


def test_distributions_have_the_stated_moments():
    w, Y = workloads.make("square_4096")                      # N(0,1) times a per-column scale in [0.01, 1]
    s = Y.std(axis=0)
    assert 0.009 < s.min() < 0.02 and 0.9 < s.max() < 1.05
    assert abs(np.log10(s).mean() + 1.0) < 0.05               # log-uniform over two decades
    w, Y = workloads.make("paper_1000x10000")                 # U(0,1) as in the paper's timing runs (Sec. 6.1)
    assert Y.min() >= 0.0 and Y.max() < 1.0 and abs(Y.mean() - 0.5) < 1e-3
    Y = workloads.generate((2000, 50), "laplace", 7)
    assert abs(np.abs(Y).mean() - 1.0) < 0.02 and abs(Y.var() - 2.0) < 0.1
    Y = workloads.generate((2000, 50), "normal", 7)
    assert abs(Y.mean()) < 0.01 and abs(Y.std() - 1.0) < 0.01
