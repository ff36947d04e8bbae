"""The device planner's chunk count ceil(len / c) without an integer division (CPU check of the arithmetic).

The kernels that plan the chunks of per-sequence lengths (Eq. 6's chunks, one list for all sequences) estimate
the quotient with the float reciprocal of the chunk length and correct it by one step either way.  That is exact
for lengths and chunk lengths below 2^23 with chunk lengths of at least 32; this test replays the same float32
arithmetic in numpy on random and adversarial pairs, with the reciprocal off by an ulp either way as well
(a hardware reciprocal need not be correctly rounded)."""
import numpy as np
import pytest


def _chunks_fast(length, c, ulp):
    x = (length + c - 1).astype(np.int64)
    rc = (np.float32(1.0) / c.astype(np.float32)).astype(np.float32)
    if ulp:
        rc = np.nextafter(rc, np.float32(np.inf if ulp > 0 else -np.inf)).astype(np.float32)
    q = (x.astype(np.float32) * rc).astype(np.float32).astype(np.int64)   # float -> int truncates, as on the device
    r = x - q * c
    return q + (r >= c) - (r < 0)


@pytest.mark.parametrize("ulp", [0, 1, -1])
def test_chunk_count_by_reciprocal_is_exact_below_2_to_23(ulp):
    rng = np.random.default_rng(23 + ulp)
    top = (1 << 23) - 1
    for kind in range(6):
        n = 200_000
        c = 32 * (rng.integers(1, 300, n) if kind % 2 == 0 else rng.integers(1, 1 << 18, n))
        c = np.minimum(c, (1 << 23) - 32)
        if kind < 2:
            length = rng.integers(0, 1 << 23, n)
        elif kind < 4:                                 # around exact multiples of c: where a floor can tip over
            length = rng.integers(0, 1 << 19, n) * c + rng.integers(-2, 3, n)
        else:
            length = rng.integers(0, 1 << 12, n) * c // 7
        length = np.clip(length, 0, top)
        assert np.array_equal(_chunks_fast(length, c, ulp), (length + c - 1) // c)
    # the corners
    length = np.array([0, 1, 31, 32, 33, top, top, top], dtype=np.int64)
    c = np.array([32, 32, 32, 32, 32, 32, (1 << 23) - 32, 64], dtype=np.int64)
    assert np.array_equal(_chunks_fast(length, c, ulp), (length + c - 1) // c)
