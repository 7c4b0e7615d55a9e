"""Oracle: Philox4x32-R and the dropout keep-mask.  TEST INFRASTRUCTURE ONLY.

Two implementations live here on purpose:
  * thin ctypes wrappers over oracle/philox_oracle.c (scalar C, used at the
    sizes of the paper's workloads), and
  * `philox4x32_py` / `dropout_mask_py`, a second evaluation of the same
    definitions with Python's unbounded integers, used by the pin tests on
    tiny inputs to cross-check the C code.

The paper (Sec. 2.3) only names Philox and cites its publication; the round
function and constants come from that publication and are pinned by its
known-answer vectors.  The keep-mask layout is this build's reading of the
paper's "one bit per element" (Sec. 6.1, Sec. 7.2).
"""
import ctypes
import os

import numpy as np

from . import build_oracle

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.build(force=False)
        L = ctypes.CDLL(path)
        u64, u32p, u64p = ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint64)
        L.oracle_philox4x32.argtypes = [u32p, u32p, ctypes.c_int, u32p]
        L.oracle_philox4x32.restype = None
        L.oracle_philox_raw.argtypes = [u64, u64, u64, ctypes.c_int, ctypes.c_void_p]
        L.oracle_philox_raw.restype = None
        L.oracle_keep_threshold.argtypes = [ctypes.c_float, u64p]
        L.oracle_keep_threshold.restype = ctypes.c_int
        L.oracle_mask_words.argtypes = [ctypes.c_int] * 3
        L.oracle_mask_words.restype = u64
        L.oracle_mask_philox_calls.argtypes = [ctypes.c_int] * 3
        L.oracle_mask_philox_calls.restype = u64
        L.oracle_dropout_mask_rounds.argtypes = [u64, u64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_float, ctypes.c_int, ctypes.c_void_p]
        L.oracle_dropout_mask_rounds.restype = ctypes.c_int
        L.oracle_dropout_mask_bits.argtypes = [u64, u64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.oracle_dropout_mask_bits.restype = ctypes.c_int
        L.oracle_keep_threshold_bits.argtypes = [ctypes.c_float, ctypes.c_int, u64p]
        L.oracle_keep_threshold_bits.restype = ctypes.c_int
        L.oracle_mask_philox_calls_bits.argtypes = [ctypes.c_int] * 4
        L.oracle_mask_philox_calls_bits.restype = u64
        L.oracle_popcount_words.argtypes = [ctypes.c_void_p, u64]
        L.oracle_popcount_words.restype = u64
        L.oracle_num_threads.argtypes = []
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def philox4x32(ctr, key, rounds=10):
    """One Philox-4x32 block (C oracle): 4 counter words, 2 key words -> 4 words."""
    c = (ctypes.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (ctypes.c_uint32 * 4)()
    lib().oracle_philox4x32(c, k, int(rounds), o)
    return [int(v) for v in o]


def philox_raw(seed, first_counter, ncalls, rounds=10):
    """uint32[ncalls, 4]: row i = Philox(key = seed, counter = first_counter + i)."""
    out = np.empty((int(ncalls), 4), dtype=np.uint32)
    lib().oracle_philox_raw(int(seed) & (2**64 - 1), int(first_counter) & (2**64 - 1),
                            int(ncalls), int(rounds), out.ctypes.data)
    return out


def keep_threshold(p):
    """T = floor((1 - p) * 2^32) from the float32 value of p; p in [0, 1)."""
    T = ctypes.c_uint64(0)
    rc = lib().oracle_keep_threshold(ctypes.c_float(p), ctypes.byref(T))
    if rc != 0:
        raise ValueError("p must satisfy 0 <= p < 1")
    return int(T.value)


def mask_words(B, H, S):
    return int(lib().oracle_mask_words(B, H, S))


def mask_philox_calls(B, H, S):
    return int(lib().oracle_mask_philox_calls(B, H, S))


def dropout_mask(seed, offset, B, H, S, p, rounds=10):
    """Keep-mask words, uint64[B, H, T, T, 16] with T = ceil(S/32): 32 x 32 tiles of 16 words;
    bit l of word e of tile (qt, kt) = element (32 qt + l%32, 32 kt + 8 (e/4) + 4 (l/32) + e%4)."""
    T = (S + 31) // 32
    out = np.zeros((B, H, T, T, 16), dtype=np.uint64)
    rc = lib().oracle_dropout_mask_rounds(int(seed) & (2**64 - 1), int(offset) & (2**64 - 1),
                                          B, H, S, ctypes.c_float(p), int(rounds), out.ctypes.data)
    if rc != 0:
        raise ValueError("invalid mask arguments")
    return out


def keep_threshold_bits(p, bits):
    """Tb = floor((1 - p) * 2^bits) from the float32 value of p; bits in {8, 16, 32}."""
    T = ctypes.c_uint64(0)
    if lib().oracle_keep_threshold_bits(ctypes.c_float(p), int(bits), ctypes.byref(T)) != 0:
        raise ValueError("p must satisfy 0 <= p < 1 and bits must be 8, 16 or 32")
    return int(T.value)


def mask_philox_calls_bits(B, H, S, bits):
    return int(lib().oracle_mask_philox_calls_bits(B, H, S, int(bits)))


def dropout_mask_bits(seed, offset, B, H, S, p, bits, rounds=10):
    """Keep-mask drawn with `bits` random bits per element (8, 16 or 32): same layout as
    dropout_mask; words in groups of 4*32/bits, field e/4 of output word e%4 decides word e."""
    T = (S + 31) // 32
    out = np.zeros((B, H, T, T, 16), dtype=np.uint64)
    rc = lib().oracle_dropout_mask_bits(int(seed) & (2**64 - 1), int(offset) & (2**64 - 1), B, H, S,
                                        ctypes.c_float(p), int(rounds), int(bits), out.ctypes.data)
    if rc != 0:
        raise ValueError("invalid mask arguments")
    return out


def popcount(words):
    w = np.ascontiguousarray(words, dtype=np.uint64)
    return int(lib().oracle_popcount_words(w.ctypes.data, w.size))


def num_threads():
    return int(lib().oracle_num_threads())


def unpack_keep(words, S):
    """bool[..., S, S] keep matrix from mask words [..., T, T, 16] (T = ceil(S/32))."""
    w = np.ascontiguousarray(words, dtype="<u8")
    T = w.shape[-3]
    lead = w.shape[:-3]
    bits = np.unpackbits(w.view(np.uint8), axis=-1, bitorder="little")       # [..., qt, kt, 16*64]
    bits = bits.reshape(lead + (T, T, 4, 4, 2, 32))                          # qt, kt, e/4, e%4, l/32, l%32
    nd = len(lead)
    # row = (qt, l%32); column = (kt, e/4, l/32, e%4)
    order = tuple(range(nd)) + (nd + 0, nd + 5, nd + 1, nd + 2, nd + 4, nd + 3)
    full = bits.transpose(order).reshape(lead + (32 * T, 32 * T))
    return full[..., :S, :S].astype(bool)


def unpack_keep_rows(tile_rows, S):
    """bool[..., 32, S] for one row of tiles: words [..., T, 16] of a fixed qt."""
    w = np.ascontiguousarray(tile_rows, dtype="<u8")
    T = w.shape[-2]
    lead = w.shape[:-2]
    bits = np.unpackbits(w.view(np.uint8), axis=-1, bitorder="little").reshape(lead + (T, 4, 4, 2, 32))
    nd = len(lead)
    order = tuple(range(nd)) + (nd + 4, nd + 0, nd + 1, nd + 3, nd + 2)
    return bits.transpose(order).reshape(lead + (32, 32 * T))[..., :S].astype(bool)


# ---------------------------------------------------------------------------
# Second evaluation with Python integers (tiny inputs only).
# ---------------------------------------------------------------------------
_M0, _M1 = 0xD2511F53, 0xCD9E8D57
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_py(ctr, key, rounds=10):
    c0, c1, c2, c3 = [int(v) & _MASK32 for v in ctr]
    k0, k1 = [int(v) & _MASK32 for v in key]
    for _ in range(rounds):
        p0 = _M0 * c0
        p1 = _M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & _MASK32, p1 & _MASK32, \
                         ((p0 >> 32) ^ c3 ^ k1) & _MASK32, p0 & _MASK32
        k0 = (k0 + _W0) & _MASK32
        k1 = (k1 + _W1) & _MASK32
    return [c0, c1, c2, c3]


def dropout_mask_py(seed, offset, B, H, S, p, rounds=10, bits=32):
    """Element-by-element evaluation of the mask definition (no grouping)."""
    thr = int((1.0 - float(np.float32(p))) * float(2**bits))  # IEEE double, truncation = floor
    E = 4 * (32 // bits)
    T = (S + 31) // 32
    out = np.zeros((B, H, T, T, 16), dtype=np.uint64)
    flat = out.reshape(-1)
    key = [seed & _MASK32, (seed >> 32) & _MASK32]
    for w in range(flat.size):
        word = 0
        e, kt, qt = w % 16, (w // 16) % T, (w // (16 * T)) % T
        for l in range(64):
            i = 32 * qt + l % 32
            j = 32 * kt + 8 * (e // 4) + 4 * (l // 32) + e % 4
            if i >= S or j >= S:
                continue
            n = (offset + 64 * (w // E) + l) % 2**64
            x = philox4x32_py([n & _MASK32, n >> 32, 0, 0], key, rounds)[(w % E) % 4]
            x = (x >> (bits * ((w % E) // 4))) & (2**bits - 1)
            if x < thr:
                word |= 1 << l
        flat[w] = word
    return out
