"""Counter-based 64-bit generator (splitmix64) and integer draws, vectorised with numpy.

splitmix64 is fully specified by three constants and is stateless per element: element i
of the stream with seed S is mix(S + (i+1)*GAMMA mod 2^64).  That makes it reproducible
across languages and lets huge tensors be drawn in one vectorised pass.  Integers in
[lo, hi] are lo + (u64 mod (hi-lo+1)); the modulo bias (< 2^-32 here) is irrelevant for
test inputs and keeps the definition trivial to re-implement.
"""
from __future__ import annotations

import numpy as np

_GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1


def _mix_py(z: int) -> int:
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def splitmix64_scalar(seed: int, n: int) -> list:
    """Pure-Python stream (arbitrary-precision ints): the second implementation the
    vectorised one is cross-checked against."""
    out, s = [], seed & _MASK
    for _ in range(n):
        s = (s + _GAMMA) & _MASK
        out.append(_mix_py(s))
    return out


def splitmix64_stream(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """Elements [offset, offset+n) of the splitmix64 stream for `seed`, as uint64."""
    with np.errstate(over="ignore"):
        idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        z = np.uint64(seed & _MASK) + idx * np.uint64(_GAMMA)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
        z = z ^ (z >> np.uint64(31))
    return z


def tensor_seed(base_seed: int, config_id: int, op_index: int, kind: str) -> int:
    """Per-tensor stream seed: one splitmix64 mixing step over (base, config, op, kind).

    kind is one of 'x', 'w', 'bias', 'm', 's', 'res', 'acc', 'act'.
    """
    kinds = {"x": 1, "w": 2, "bias": 3, "m": 4, "s": 5, "res": 6, "acc": 7, "act": 8}
    v = (base_seed & _MASK)
    for part in (config_id + 1, op_index + 1, kinds[kind]):
        v = _mix_py((v + part * _GAMMA) & _MASK)
    return v


def randint_array(seed: int, shape, lo: int, hi: int, dtype) -> np.ndarray:
    """Integers uniform in [lo, hi] (inclusive), drawn in C order, chunked to bound memory."""
    n = int(np.prod(shape)) if len(shape) else 1
    span = hi - lo + 1
    out = np.empty(n, dtype=dtype)
    chunk = 1 << 24
    for start in range(0, n, chunk):
        cnt = min(chunk, n - start)
        u = splitmix64_stream(seed, cnt, offset=start)
        out[start:start + cnt] = (u % np.uint64(span)).astype(np.int64) + lo
    return out.reshape(shape)
