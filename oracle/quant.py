"""CPU oracle -- TEST INFRASTRUCTURE ONLY: the quantization operators of the paper's generic
quantization flow (Section 4.2) with selectable rounding.

  simQ(x, beta, sigma, rho) = clip(round(x / rho * 2^(beta - sigma))) * rho / 2^(beta - sigma)   ("Annotate")
  Q(x, rho, beta, sigma)    = cast(clip(round(x / rho * 2^(beta - sigma)), qtype))                ("Realize")

and the rounding strategies the section names: nearest, floor, ceiling, stochastic.  The same
strategies apply to the integer requantization `acc / 2^s` that a realized conv ends with.

Readings (the section is terse): beta = bits of the target type, sigma = the bits that do not
carry magnitude (1 for a signed type, 0 for an unsigned one: the section lets a scheme choose
between signed and unsigned integers), rho = the range that maps onto the full scale; the clip
is symmetric for a signed type, +-(2^(beta-1) - 1), and [0, 2^beta - 1] for an unsigned one;
"nearest" breaks ties toward +infinity, as the integer path does.  Floating point decides the integer code here, so the decision is taken in the kernel's
precision: fp32, in the operation order written above (x / rho, then times the power of two,
then the rounding rule) -- numpy float32 performs the same IEEE operations.

Stochastic rounding draws from Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random
numbers: as easy as 1, 2, 3", SC'11), a counter-based generator: element e of a tensor (its
linear index in the layout the caller names) uses word e mod 4 of the block with counter
(e div 4, 0, 0, 0) and key (seed low word, seed high word).
"""
from __future__ import annotations

import numpy as np

NEAREST, FLOOR, CEIL, STOCHASTIC = 0, 1, 2, 3

_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter, key):
    """counter: uint32 array [..., 4]; key: (k0, k1).  Returns uint32 [..., 4]."""
    c = [np.asarray(counter[..., i], dtype=np.uint64) for i in range(4)]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c[0]                  # 64-bit products of 32-bit operands
        p1 = _M1 * c[2]
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK
        c = [hi1 ^ c[1] ^ np.uint64(k0), lo1, hi0 ^ c[3] ^ np.uint64(k1), lo0]
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack([x.astype(np.uint32) for x in c], axis=-1)


def random_words(index, seed: int) -> np.ndarray:
    """One 32-bit word per element index (any integer array), as defined in the module header."""
    idx = np.asarray(index, dtype=np.uint64)
    blk = idx >> np.uint64(2)
    ctr = np.zeros(idx.shape + (4,), dtype=np.uint32)
    ctr[..., 0] = (blk & _MASK).astype(np.uint32)
    ctr[..., 1] = (blk >> np.uint64(32)).astype(np.uint32)
    out = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    return np.take_along_axis(out, (idx & np.uint64(3)).astype(np.int64)[..., None], axis=-1)[..., 0]


def rshift_mode(acc, s: int, mode: int = NEAREST, seed: int = 0, index=None) -> np.ndarray:
    """acc / 2^s rounded by `mode`, on int64.  Stochastic: floor((acc + u) / 2^s) with u the low s
    bits of the element's random word, i.e. rounds up with probability frac(acc / 2^s)."""
    a = np.asarray(acc, dtype=np.int64)
    assert 0 <= s <= 31
    if s == 0:
        return a.copy()
    d = np.int64(1) << np.int64(s)
    if mode == NEAREST:
        return np.floor_divide(a + (d >> np.int64(1)), d)
    if mode == FLOOR:
        return np.floor_divide(a, d)
    if mode == CEIL:
        return -np.floor_divide(-a, d)
    if mode == STOCHASTIC:
        u = random_words(index, seed).astype(np.int64) & (d - np.int64(1))
        return np.floor_divide(a + u, d)
    raise ValueError(mode)


def _round_f32(t: np.ndarray, mode: int, seed: int, index) -> np.ndarray:
    t = t.astype(np.float32)
    if mode == NEAREST:
        return np.floor(t + np.float32(0.5))
    if mode == FLOOR:
        return np.floor(t)
    if mode == CEIL:
        return np.ceil(t)
    if mode == STOCHASTIC:
        u = (random_words(index, seed) >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)
        return np.floor(t + u)
    raise ValueError(mode)


def quantize_codes(x, rho: float, beta: int, sigma: int, mode: int = NEAREST, seed: int = 0) -> np.ndarray:
    """clip(round(x / rho * 2^(beta - sigma))) as float32 integers, element index = position in x.ravel()."""
    x32 = np.asarray(x).astype(np.float32)
    t = (x32 / np.float32(rho)) * np.float32(2.0 ** (beta - sigma))
    idx = np.arange(x32.size, dtype=np.uint64).reshape(x32.shape)
    q = _round_f32(t, mode, seed, idx)
    if sigma == 0:                                   # an unsigned target type; what is not positive is the code +0
        return np.where(q > 0, np.minimum(q, np.float32(2 ** beta - 1)), np.float32(0)).astype(np.float32)
    lim = np.float32(2 ** (beta - 1) - 1)
    return np.clip(q, -lim, lim)


def Q(x, rho: float, beta: int, sigma: int, mode: int = NEAREST, seed: int = 0) -> np.ndarray:
    """The realized quantization operator; beta <= 8 gives int8 codes, uint8 ones for an unsigned type (sigma 0)."""
    assert 2 <= beta <= 8
    return quantize_codes(x, rho, beta, sigma, mode, seed).astype(np.uint8 if sigma == 0 else np.int8)


def simQ(x, beta: int, sigma: int, rho: float, mode: int = NEAREST, seed: int = 0) -> np.ndarray:
    """Simulated quantization on the unquantized type (fp32 in, fp32 out)."""
    q = quantize_codes(x, rho, beta, sigma, mode, seed)
    return (q * np.float32(rho)) / np.float32(2.0 ** (beta - sigma))


def qconv2d_requant_mode(x, w, *, stride=(1, 1), pad=(0, 0), bias=None, residual=None, residual_lshift: int = 0,
                         out_rshift: int = 0, relu_flag=False, mode: int = NEAREST, seed: int = 0) -> np.ndarray:
    """The realized int8 conv with a rounding strategy: exact sum -> [bias] -> [+res*2^l] ->
    acc / 2^s by `mode` -> clip +-127 -> [relu] -> int8.  The element index of the stochastic
    draw is the position in the NHWC output, ((n*Ho + p)*Wo + q)*K + k."""
    import oracle as O
    acc = O.conv2d_int(x, w, stride, pad)
    if bias is not None:
        acc = O.bias_add_int(acc, bias)
    if residual is not None:
        acc = O.add_lshift_int(acc, residual, residual_lshift)
    O.assert_fits_i32(acc)
    n, k, ho, wo = acc.shape
    nn, kk, pp, qq = np.meshgrid(np.arange(n), np.arange(k), np.arange(ho), np.arange(wo), indexing="ij")
    index = ((nn * ho + pp) * wo + qq) * k + kk
    q = rshift_mode(acc, out_rshift, mode, seed, index)
    q = O.clip_int(q, -127, 127)
    if relu_flag:
        q = O.relu_int(q)
    return O.cast_i8(q)
