"""The entry point that allocates nothing (dsspk_colsum_noalloc: slab sums in a buffer that is part of the library
image) against the existing dsspk_colsum with a caller-provided workspace: same kernels, so the same bits, on two calls
in a row, the second with a smaller input (the shared buffer keeps the first call's contents)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_1908_11848_amd import binding as B               # noqa: E402
from gpu_util import dev, empty, host, rel_l2, stream_ptr     # noqa: E402

MAX_N = 4096            # DSSPK_COLSUM_NOALLOC_MAX_N
ETOOBIG = -2            # DSSPK_NOALLOC_ETOOBIG


def both(x):
    L = B.lib()
    s = stream_ptr()
    M, N = x.shape
    X = dev(x)
    need = L.dsspk_colsum_scratch_floats(M, N)
    scratch = empty(max(1, need))
    want, got = empty(N), empty(N)
    assert L.dsspk_colsum(s, X.data_ptr(), want.data_ptr(), scratch.data_ptr() if need else None, M, N) == 0
    assert L.dsspk_colsum_noalloc(s, X.data_ptr(), got.data_ptr(), M, N) == 0
    return host(want), host(got)


def test_colsum_noalloc_matches_colsum_on_two_calls_in_a_row():
    g = np.random.default_rng(77)
    first = g.standard_normal((131072, 64)).astype(np.float32)          # 256 slabs of 512 rows
    second = g.standard_normal((5000, 37)).astype(np.float32)           # fewer, shorter slabs, ragged columns
    third = g.standard_normal((300, 100)).astype(np.float32)            # short matrix: one pass, no slab sums at all
    for x in (first, second, third, first):
        want, got = both(x)
        assert np.array_equal(want, got)
        assert rel_l2(got, x.astype(np.float64).sum(0)) < 2e-6           # and both are the column sums
    L = B.lib()
    x = dev(np.zeros((2048, 8), dtype=np.float32)); out = empty(MAX_N + 1)
    assert L.dsspk_colsum_noalloc(stream_ptr(), x.data_ptr(), out.data_ptr(), 2, MAX_N + 1) == ETOOBIG   # rejected on the host
    assert L.dsspk_colsum_noalloc(stream_ptr(), None, out.data_ptr(), 2, 8) == -1
    wide = g.standard_normal((1500, MAX_N)).astype(np.float32)           # the widest matrix the fixed buffer serves
    want, got = both(wide)
    assert np.array_equal(want, got)
