"""Counter-based random columns: value = mix(seed, column id, row index).

Written with torch tensor operations only, so the same function fills a column
on the host (for the oracle at small sizes) or directly in HBM (for full-size
runs) and yields identical bits on both: every step is either wrapping 64-bit
integer arithmetic or one correctly rounded f64 operation on exact inputs.

Because a value depends only on (seed, column, row), generation is order
independent and can be done in chunks.
"""
import torch

_M64 = (1 << 64) - 1


def _s64(x):
    """Python int (mod 2^64) -> the signed value torch.int64 holds for it."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_MUL1 = _s64(0xBF58476D1CE4E5B9)
_MUL2 = _s64(0x94D049BB133111EB)


def _lsr(z, k):
    """Logical shift right of an int64 tensor (torch's >> is arithmetic)."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def bits64(seed, column, start, count, device="cpu"):
    """`count` 64-bit words for rows start..start+count-1 of one column."""
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    key = _s64((seed * 0xD1342543DE82EF95 + (column + 1) * 0xA0761D6478BD642F) & _M64)
    z = i * _GOLDEN + key
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    z = z ^ _lsr(z, 31)
    return z


def unit_f64(seed, column, start, count, device="cpu"):
    """Uniform doubles in [0,1): top 53 bits times 2^-53 (exact)."""
    z = bits64(seed, column, start, count, device)
    return _lsr(z, 11).to(torch.float64) * (1.0 / 9007199254740992.0)


def uniform_f64(seed, column, start, count, lo, hi, device="cpu"):
    """lo + (hi-lo)*u, u in [0,1): two rounded f64 operations."""
    u = unit_f64(seed, column, start, count, device)
    return u * (hi - lo) + lo


def uniform_int(seed, column, start, count, lo, hi, device="cpu"):
    """Integer uniform on lo..hi inclusive, returned as int64."""
    u = unit_f64(seed, column, start, count, device)
    m = hi - lo + 1
    k = torch.floor(u * float(m)).to(torch.int64)
    k = torch.clamp(k, max=m - 1)
    return k + lo
