"""Helpers for the tests: numpy-side number formats (independent of the oracle's own)."""
import numpy as np


def f16_bits_to_f64(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def f64_to_f16_bits(x):
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float16).view(np.uint16)


def bf16_bits_to_f64(bits):
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).astype(np.float64)


def bits_to_f64(bits, dtype):
    return f16_bits_to_f64(bits) if dtype == 1 else bf16_bits_to_f64(bits)


def ulp_distance_16(a_bits, b_bits):
    """Distance in units in the last place between two arrays of 16-bit float patterns
    (sign-magnitude mapped to a monotone integer line)."""
    def key(u):
        u = np.asarray(u, dtype=np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    return np.abs(key(a_bits) - key(b_bits))


def unpack_int(buf, n, bits):
    """Codes from a packed little-endian bit stream, via one big Python integer."""
    v = int.from_bytes(bytes(bytearray(buf)), "little")
    return np.array([(v >> (i * bits)) & ((1 << bits) - 1) for i in range(n)], dtype=np.uint8)


def unpack_np(buf, bits):
    """Vectorised unpack of a packed byte array (bit k of the stream = bit k%8 of byte k/8)."""
    bitsarr = np.unpackbits(np.asarray(buf, dtype=np.uint8), bitorder="little")
    bitsarr = bitsarr.reshape(-1, bits).astype(np.uint16)
    return (bitsarr << np.arange(bits, dtype=np.uint16)).sum(axis=1).astype(np.uint8)
