"""CPU oracle for the per-pass random partition of a buffer (TEST INFRASTRUCTURE).

Algorithm 1 regenerates, at the start of every pass t over buffer S_{r,k}, a
random partition {S^(t,1), ..., S^(t,M)} of the buffer into mini-batches, and
Section 2.2 requires the parts to be disjoint and to cover the buffer.  The
paper does not name a random generator, so one is fixed here (stated in
full below) that needs only 32-bit integer arithmetic and is therefore
reproducible bit for bit on any machine:

    perm = PERM(seed, b, t, N0)       a bijection of {0, ..., N0-1}
    mini-batch m (1-based) = perm[(m-1) n : min(m n, N0)]

``b`` is the 0-based count of buffers processed so far, ``t`` the 1-based pass
(t = 0 is used for the "fixed partition" setting of Section 3.1.1).

Definition (all values uint32, arithmetic modulo 2^32):

    mix(x):  x ^= x >> 16;  x *= 0x7FEB352D;  x ^= x >> 15;
             x *= 0x846CA68B;  x ^= x >> 16
    bits = number of bits needed to write N0-1 (0 when N0 = 1)
    h    = max(1, ceil(bits / 2));  mask = 2^h - 1        (block width 2h bits)
    a    = mix(seed_lo ^ 0x9E3779B9);  a = mix(a ^ seed_hi)
    a    = mix(a + b);  a = mix(a ^ t)
    key_i = mix(a + i * 0x9E3779B9)                for i = 0 .. 7
    E(x): (L, R) = (x >> h, x & mask)
          for i = 0 .. 7:  (L, R) = (R, L ^ (mix(R ^ key_i) & mask))
          return (L << h) | R
    perm[j] = first element of E(j), E(E(j)), ... that is < N0

E is a balanced Feistel network, hence a bijection of {0, ..., 2^(2h) - 1};
following its cycles until they re-enter {0, ..., N0-1} ("cycle walking")
restricts it to a bijection of that set.  2^(2h) < 4 N0, so fewer than four
applications of E are needed on average.

Two independent implementations live here -- a scalar one in plain Python
integers and a vectorised numpy one -- and the tests require them to agree.
Nothing in this file is imported by the GPU library or its Python binding.
"""
from __future__ import annotations

import numpy as np

ROUNDS = 8
_M32 = 0xFFFFFFFF
_GOLD = 0x9E3779B9
_C1 = 0x7FEB352D
_C2 = 0x846CA68B


# ---------------------------------------------------------------- scalar form
def mix_scalar(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * _C1) & _M32
    x ^= x >> 15
    x = (x * _C2) & _M32
    x ^= x >> 16
    return x


def half_width(N0: int) -> int:
    bits = (N0 - 1).bit_length()
    return max(1, (bits + 1) // 2)


def round_keys(seed: int, b: int, t: int) -> list[int]:
    seed_lo, seed_hi = seed & _M32, (seed >> 32) & _M32
    a = mix_scalar(seed_lo ^ _GOLD)
    a = mix_scalar(a ^ seed_hi)
    a = mix_scalar((a + b) & _M32)
    a = mix_scalar(a ^ (t & _M32))
    return [mix_scalar((a + i * _GOLD) & _M32) for i in range(ROUNDS)]


def feistel_scalar(x: int, keys: list[int], h: int) -> int:
    mask = (1 << h) - 1
    L, R = x >> h, x & mask
    for k in keys:
        L, R = R, L ^ (mix_scalar(R ^ k) & mask)
    return (L << h) | R


def feistel_inverse_scalar(y: int, keys: list[int], h: int) -> int:
    """Inverse of feistel_scalar, used only to check the network really is one."""
    mask = (1 << h) - 1
    L, R = y >> h, y & mask
    for k in reversed(keys):
        L, R = R ^ (mix_scalar(L ^ k) & mask), L
    return (L << h) | R


def perm_scalar(seed: int, b: int, t: int, N0: int) -> list[int]:
    if N0 <= 0:
        return []
    h = half_width(N0)
    keys = round_keys(seed, b, t)
    out = []
    for j in range(N0):
        x = feistel_scalar(j, keys, h)
        while x >= N0:
            x = feistel_scalar(x, keys, h)
        out.append(x)
    return out


# ------------------------------------------------------------ vectorised form
def _mix_vec(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.uint32, copy=True)
    x ^= x >> np.uint32(16)
    x *= np.uint32(_C1)
    x ^= x >> np.uint32(15)
    x *= np.uint32(_C2)
    x ^= x >> np.uint32(16)
    return x


def _feistel_vec(x: np.ndarray, keys: list[int], h: int) -> np.ndarray:
    mask = np.uint32((1 << h) - 1)
    hh = np.uint32(h)
    L, R = x >> hh, x & mask
    for k in keys:
        L, R = R, L ^ (_mix_vec(R ^ np.uint32(k)) & mask)
    return (L << hh) | R


def perm(seed: int, b: int, t: int, N0: int) -> np.ndarray:
    """PERM(seed, b, t, N0) as an int32 array of length N0."""
    if N0 <= 0:
        return np.empty(0, dtype=np.int32)
    if N0 > (1 << 30):
        raise ValueError("N0 above 2^30 is outside the supported range")
    h = half_width(N0)
    keys = round_keys(seed, b, t)
    with np.errstate(over="ignore"):
        x = _feistel_vec(np.arange(N0, dtype=np.uint32), keys, h)
        todo = np.nonzero(x >= N0)[0]
        while todo.size:
            x[todo] = _feistel_vec(x[todo], keys, h)
            todo = todo[x[todo] >= N0]
    return x.astype(np.int32)


def minibatches(perm_arr: np.ndarray, n: int) -> list[np.ndarray]:
    """Split a permutation into consecutive mini-batch index sets of size n (last may be short)."""
    N0 = len(perm_arr)
    return [perm_arr[s:min(s + n, N0)] for s in range(0, N0, n)]
