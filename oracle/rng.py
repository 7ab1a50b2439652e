"""Counter-based random numbers for T > 0 (test infrastructure; see package docstring).

The paper fixes no randomness source.  Both this oracle and the HIP path
implement the same stateless generator so that they take the same decisions:
a splitmix64-style finaliser chained over (seed, cycle, node, draw); the
uniform is the top 23 bits, centred in its cell so that it is never 0 or 1
and every value is exact in float32.
"""
import numpy as np

_M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
GUMBEL_BASE = 1 << 32          # draw index of vocabulary entry v in the bonus draw is GUMBEL_BASE + v


def mix64(x):
    """splitmix64 finaliser on python ints or uint64 arrays."""
    if isinstance(x, np.ndarray):
        x = x.astype(np.uint64)
        with np.errstate(over="ignore"):
            x = x ^ (x >> np.uint64(30))
            x = x * np.uint64(0xBF58476D1CE4E5B9)
            x = x ^ (x >> np.uint64(27))
            x = x * np.uint64(0x94D049BB133111EB)
            x = x ^ (x >> np.uint64(31))
        return x
    x &= _M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _M64
    x ^= x >> 31
    return x


def _stream(seed: int, cycle: int, node: int) -> int:
    s = mix64((seed + GOLDEN) & _M64)
    s = mix64((s + cycle) & _M64)
    s = mix64((s + node) & _M64)
    return s


def uniform01(seed: int, cycle: int, node: int, draw) -> np.ndarray:
    """u in (0,1) as float32: ((bits >> 41) + 0.5) * 2**-23; `draw` int or int array."""
    s = _stream(seed, cycle, node)
    d = np.asarray(draw, dtype=np.uint64)
    with np.errstate(over="ignore"):
        bits = mix64(np.atleast_1d(d + np.uint64(s)))
    top = (bits >> np.uint64(41)).astype(np.float32)
    u = (top + np.float32(0.5)) * np.float32(2.0 ** -23)
    return u if np.ndim(draw) else u[0]


def gumbel(seed: int, cycle: int, node: int, vocab: int) -> np.ndarray:
    """Standard Gumbel noise per vocabulary entry, float32: -log(-log(u_v))."""
    u = uniform01(seed, cycle, node, np.arange(vocab, dtype=np.uint64) + np.uint64(GUMBEL_BASE))
    return (-np.log(-np.log(u.astype(np.float32)))).astype(np.float32)
