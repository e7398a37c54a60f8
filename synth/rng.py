"""Counter-based random numbers: splitmix64 -> uniform -> Box-Muller normal.

Every value is a pure function of (seed, index), so a tensor of any size can be
generated in vectorised chunks and the i-th value never depends on how many
were asked for.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """u64 outputs number start .. start+count-1 of the splitmix64 stream of `seed`."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, start: int, count: int) -> np.ndarray:
    """Doubles in (0, 1]: top 53 bits of the stream, plus one, over 2^53."""
    u = splitmix64(seed, start, count) >> np.uint64(11)
    return (u.astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal(seed: int, count: int, chunk: int = 1 << 22) -> np.ndarray:
    """`count` standard normals as float64.  Value 2i and 2i+1 come from the
    uniform pair (2i, 2i+1) by Box-Muller (cosine branch first, then sine)."""
    out = np.empty(count, dtype=np.float64)
    pairs = (count + 1) // 2
    done = 0
    while done < pairs:
        n = min(chunk, pairs - done)
        u = uniform01(seed, 2 * done, 2 * n)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        th = (2.0 * np.pi) * u[1::2]
        z = np.empty(2 * n, dtype=np.float64)
        z[0::2] = r * np.cos(th)
        z[1::2] = r * np.sin(th)
        lo = 2 * done
        hi = min(count, lo + 2 * n)
        out[lo:hi] = z[: hi - lo]
        done += n
    return out


def labels_uniform(seed: int, count: int, classes: int) -> np.ndarray:
    """int32 labels: stream value modulo `classes`."""
    return (splitmix64(seed, 0, count) % np.uint64(classes)).astype(np.int32)
