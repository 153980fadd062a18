"""Counter-based random numbers: value i of stream s under a seed is a pure
function of (seed, s, i), so any slice can be regenerated anywhere."""
import numpy as np

_U64 = np.uint64
_G1 = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)


def mix64(x):
    """64-bit avalanche mix (the splitmix64 finaliser) on a uint64 array or scalar."""
    with np.errstate(over="ignore"):
        x = np.asarray(x, dtype=_U64)
        x = (x ^ (x >> _U64(30))) * _M1
        x = (x ^ (x >> _U64(27))) * _M2
        return x ^ (x >> _U64(31))


def _stream_base(seed, stream):
    with np.errstate(over="ignore"):
        s = mix64(_U64(seed) * _G1 + _U64(0x51ED270B))
        return mix64(s ^ (_U64(stream) * _M2 + _G1))


def raw64(seed, stream, n, start=0):
    """uint64[n]: values start..start+n-1 of the given stream."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + n, dtype=_U64)
        return mix64(_stream_base(seed, stream) + idx * _G1)


def uniform01(seed, stream, n, start=0):
    """float64[n] in the open interval (0, 1)."""
    r = raw64(seed, stream, n, start)
    return ((r >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed, stream, n, std=1.0):
    """float64[n] ~ N(0, std^2) by Box-Muller on two sub-streams."""
    u1 = uniform01(seed, 2 * stream, n)
    u2 = uniform01(seed, 2 * stream + 1, n)
    return std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def randint(seed, stream, n, lo, hi):
    """int64[n] uniform on [lo, hi)."""
    u = uniform01(seed, stream, n)
    return (lo + np.floor(u * (hi - lo))).astype(np.int64).clip(lo, hi - 1)


class Bijection:
    """A keyed permutation of [0, size).  Built from steps that are each
    invertible on n-bit words (add key, multiply by an odd constant, xor with a
    right shift); sizes that are not powers of two use cycle walking."""

    def __init__(self, size, seed, key=0):
        size = int(size)
        assert size >= 1
        self.size = size
        self.bits = max(1, (size - 1).bit_length())
        self.mask = _U64((1 << self.bits) - 1)
        base = _stream_base(seed, 0xB17EC7 + int(key))
        ks = mix64(base + np.arange(1, 9, dtype=_U64) * _G1)
        self.add = [ks[i] & self.mask for i in range(4)]
        self.mul = [(ks[4 + i] | _U64(1)) & self.mask for i in range(4)]
        self.shift = _U64(max(1, self.bits // 2))

    def _round(self, x):
        with np.errstate(over="ignore"):
            for a, m in zip(self.add, self.mul):
                x = ((x + a) & self.mask) * m & self.mask
                x = x ^ (x >> self.shift)
        return x

    def __call__(self, i):
        x = np.asarray(i, dtype=_U64)
        assert x.size == 0 or int(x.max()) < self.size
        x = self._round(x)
        if (1 << self.bits) != self.size:
            bad = x >= _U64(self.size)
            while bad.any():
                x[bad] = self._round(x[bad])
                bad = x >= _U64(self.size)
        return x
