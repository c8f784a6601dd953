"""Test helpers written straight from the paper's identities, in Python integers.

They are NOT part of the oracle (which works on unpacked values) and not part of the
HIP library: they restate Eq. 1 (XNOR-popcount) and Eq. 2 (two subtracting bit planes)
on Python ints so the oracle's plain sums can be checked against the bit formulas the
GPU kernels rely on, and they give the bit-packing convention used at the library
boundary (channel c -> bit c%32 of word c//32, bit 1 means +1).
"""
import numpy as np


def pack_pm1(a):
    """[..., C] values in {-1,+1} -> [..., ceil(C/32)] uint32, LSB-first; pad bits 0."""
    a = np.asarray(a)
    C = a.shape[-1]
    Cw = (C + 31) // 32
    bits = np.zeros(a.shape[:-1] + (Cw * 32,), np.uint8)
    bits[..., :C] = (a > 0)
    bits = bits.reshape(a.shape[:-1] + (Cw, 32)).astype(np.uint64)
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    return (bits * weights).sum(-1).astype(np.uint32)


def pack_pm1_fast(a):
    """pack_pm1 for large tensors through numpy's packbits (bit order "little": element i of
    a group of eight goes to bit i of its byte; four such bytes read as a little-endian uint32
    are the word of pack_pm1).  C must be a multiple of 32.  Checked against pack_pm1 in
    tests/test_oracle_pins.py."""
    a = np.asarray(a)
    assert a.shape[-1] % 32 == 0
    b = np.packbits(a > 0, axis=-1, bitorder="little")
    return np.ascontiguousarray(b).view("<u4")


def unpack_pm1(words, C):
    """inverse of pack_pm1 -> int8 in {-1,+1}."""
    words = np.asarray(words, np.uint32)
    sh = np.arange(32, dtype=np.uint32)
    bits = (words[..., None] >> sh) & np.uint32(1)
    bits = bits.reshape(words.shape[:-1] + (-1,))[..., :C]
    return (bits.astype(np.int8) * 2 - 1).astype(np.int8)


def popc(x):
    return bin(int(x)).count("1")


def to_int(bits):
    """sequence of 0/1 (index 0 = LSB) -> Python int."""
    v = 0
    for i, b in enumerate(bits):
        v |= int(b) << i
    return v


def dot_xnor(a_bits, b_bits, n):
    """Eq. 1: a.b = 2*popc(a' XNOR b') - n, for a,b in {-1,+1}^n."""
    mask = (1 << n) - 1
    return 2 * popc(~(a_bits ^ b_bits) & mask) - n


def dot_two_planes(a_bits, pos, neg):
    """Eq. 2 with the constant corrected as Algorithm 1 uses it (R = C_neg - C_pos):
    a.b = popc(a' XOR b_neg) - popc(a' XOR b_pos), b = b_pos - b_neg."""
    return popc(a_bits ^ neg) - popc(a_bits ^ pos)


def dot_sign_mask(a_bits, sign, mask):
    """popc(M) - 2*popc((W xor A) & M): the sign-plane / mask-plane form."""
    return popc(mask) - 2 * popc((sign ^ a_bits) & mask)
