"""The decode kernels divide workgroup, tile and image-block indices by run-time values with one
multiplication: x / d = floor(x q / 2^32) with q = floor(2^32 / d) + 1 (q = 0 stands for d = 1),
for 0 <= x and x d < 2^32 -- the bound the host checks before it launches them.  This test checks
that rule itself, exhaustively near every multiple of d and on a grid elsewhere."""
import numpy as np


def multiplier(d: int) -> int:
    return (1 << 32) // d + 1 if d > 1 else 0


def quot(x: np.ndarray, d: int) -> np.ndarray:
    q = multiplier(d)
    return (x * np.uint64(q)) >> np.uint64(32) if q else x


def test_multiplication_equals_division_within_the_checked_bound():
    for d in list(range(1, 1300)) + [2047, 2048, 4095, 4096, 65535]:
        limit = ((1 << 32) - 1) // d                     # largest x with x d < 2^32
        top = min(limit, 1 << 22)
        mult = np.arange(0, top + 1, d, dtype=np.uint64)
        xs = np.unique(np.concatenate([mult, mult[1:] - np.uint64(1), mult + np.uint64(1),
                                       np.linspace(0, top, 4096).astype(np.uint64),
                                       np.array([limit, max(limit - 1, 0)], dtype=np.uint64)]))
        xs = xs[xs <= np.uint64(limit)]
        assert np.array_equal(quot(xs, d), xs // np.uint64(d)), d


def test_the_bound_is_needed():
    """Beyond x d < 2^32 the rule can fail: the host's check is not decoration."""
    d = 3
    x = np.array([(1 << 32) - 2], dtype=np.uint64)       # x d >= 2^32: the quotient comes out one too large
    assert int(quot(x, d)[0]) == int(x[0]) // d + 1
