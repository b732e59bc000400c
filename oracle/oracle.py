"""ctypes/numpy front end of the C oracle (oracle/neuzip_oracle.c).

Test infrastructure only.  Argument marshalling and nothing else: every step
of the method is computed inside the C file, which cites the passages of the
paper it follows.  The library is built on first use if it is missing.
"""
import ctypes
import os

import numpy as np

from . import build_oracle

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None

PROB_BITS = 12
M = 1 << PROB_BITS
CHUNK = 4096
K = 16
G = 8
RANS_L = 1 << 16
HEADER_BYTES = 64

OK, EINVAL, ENOSPACE, ECORRUPT, ESTALE = 0, -1, -2, -4, -6


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.LIB
        src = os.path.join(_HERE, "neuzip_oracle.c")
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(src):
            build_oracle.build()
        L = ctypes.CDLL(path)
        u8p, u16p, u32p, u64p = (ctypes.POINTER(t) for t in
                                 (ctypes.c_uint8, ctypes.c_uint16, ctypes.c_uint32, ctypes.c_uint64))
        u64, i32, u32 = ctypes.c_uint64, ctypes.c_int, ctypes.c_uint32
        L.nzo_split.argtypes = [u16p, u64, u8p, u8p, u8p]
        L.nzo_split.restype = None
        L.nzo_merge.argtypes = [u8p, u8p, u8p, u64, u16p]
        L.nzo_merge.restype = None
        L.nzo_truncate.argtypes = [u16p, u64, i32, u16p]
        L.nzo_truncate.restype = None
        L.nzo_signmant_bytes.argtypes = [u64, i32]
        L.nzo_signmant_bytes.restype = u64
        L.nzo_pack_signmant.argtypes = [u16p, u64, i32, u8p]
        L.nzo_pack_signmant.restype = i32
        L.nzo_histogram.argtypes = [u16p, u64, u64p]
        L.nzo_histogram.restype = None
        L.nzo_entropy.argtypes = [u64p]
        L.nzo_entropy.restype = ctypes.c_double
        L.nzo_cross_entropy.argtypes = [u64p, u16p]
        L.nzo_cross_entropy.restype = ctypes.c_double
        L.nzo_quantise.argtypes = [u64p, u16p]
        L.nzo_quantise.restype = i32
        L.nzo_quantise_guarded.argtypes = [u64p, u32, u16p]
        L.nzo_quantise_guarded.restype = i32
        L.nzo_compress_guarded.argtypes = [u16p, u64, i32, u32, u8p, u64, u64p, i32]
        L.nzo_compress_guarded.restype = i32
        L.nzo_compress_with_table.argtypes = [u16p, u64, i32, u16p, u32, u8p, u64, u64p, i32]
        L.nzo_compress_with_table.restype = i32
        L.nzo_rans_encode_step.argtypes = [u32, u32, u32, u16p, ctypes.POINTER(i32)]
        L.nzo_rans_encode_step.restype = u32
        L.nzo_rans_decode_step.argtypes = [u32, u32, u32, ctypes.c_uint16, ctypes.POINTER(i32)]
        L.nzo_rans_decode_step.restype = u32
        L.nzo_encode_chunk.argtypes = [u8p, u32, u16p, i32, i32, u32p, u16p, u16p, u32]
        L.nzo_encode_chunk.restype = i32
        L.nzo_decode_chunk.argtypes = [u8p, u32, u16p, i32, i32, u32p, u16p, u16p, u32]
        L.nzo_decode_chunk.restype = i32
        L.nzo_block_count.argtypes = [u64, u32]
        L.nzo_block_count.restype = u64
        L.nzo_block_coefficients.argtypes = [u16p, u64, u32, u8p]
        L.nzo_block_coefficients.restype = i32
        L.nzo_normalise.argtypes = [u16p, u64, u32, u8p, u16p]
        L.nzo_normalise.restype = None
        L.nzo_denormalise.argtypes = [u16p, u64, u32, u8p, u16p]
        L.nzo_denormalise.restype = None
        L.nzo_compress_blockwise.argtypes = [u16p, u64, i32, u32, u8p, u64, u64p, i32]
        L.nzo_compress_blockwise.restype = i32
        L.nzo_compress_bound.argtypes = [u64, i32]
        L.nzo_compress_bound.restype = u64
        L.nzo_compress.argtypes = [u16p, u64, i32, u8p, u64, u64p, i32]
        L.nzo_compress.restype = i32
        L.nzo_decompress.argtypes = [u8p, u64, u16p, u64, i32]
        L.nzo_decompress.restype = i32
        L.nzo_compress_f32.argtypes = [u32p, u64, u8p, u64, u64p, i32]
        L.nzo_compress_f32.restype = i32
        L.nzo_compress_f32_with_table.argtypes = [u32p, u64, u16p, u32, u8p, u64, u64p, i32]
        L.nzo_compress_f32_with_table.restype = i32
        L.nzo_compress_f16.argtypes = [u16p, u64, u16p, u32, u8p, u64, u64p, i32]
        L.nzo_compress_f16.restype = i32
        L.nzo_decompress_f16.argtypes = [u8p, u64, u16p, u64, i32]
        L.nzo_decompress_f16.restype = i32
        L.nzo_decompress_f32.argtypes = [u8p, u64, u32p, u64, i32]
        L.nzo_decompress_f32.restype = i32
        L.nzo_blob_info.argtypes = [u8p, u64, u64p, ctypes.POINTER(i32), u64p, u16p]
        L.nzo_blob_info.restype = i32
        _lib = L
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _u16(w):
    w = np.ascontiguousarray(w)
    if w.dtype != np.uint16:
        raise TypeError("bf16 words must be passed as uint16")
    return w.reshape(-1)


def split(w):
    w = _u16(w)
    n = w.size
    s, e, m = (np.empty(n, np.uint8) for _ in range(3))
    lib().nzo_split(_p(w, ctypes.c_uint16), n, _p(s, ctypes.c_uint8), _p(e, ctypes.c_uint8),
                    _p(m, ctypes.c_uint8))
    return s, e, m


def merge(s, e, m):
    s, e, m = (np.ascontiguousarray(a, dtype=np.uint8) for a in (s, e, m))
    w = np.empty(s.size, np.uint16)
    lib().nzo_merge(_p(s, ctypes.c_uint8), _p(e, ctypes.c_uint8), _p(m, ctypes.c_uint8), s.size,
                    _p(w, ctypes.c_uint16))
    return w


def truncate(w, k):
    w = _u16(w)
    out = np.empty_like(w)
    lib().nzo_truncate(_p(w, ctypes.c_uint16), w.size, k, _p(out, ctypes.c_uint16))
    return out


def signmant_bytes(n, k):
    return int(lib().nzo_signmant_bytes(n, k))


def pack_signmant(w, k):
    w = _u16(w)
    out = np.empty(signmant_bytes(w.size, k), np.uint8)
    rc = lib().nzo_pack_signmant(_p(w, ctypes.c_uint16), w.size, k, _p(out, ctypes.c_uint8))
    if rc != OK:
        raise OracleError(rc, "pack_signmant")
    return out


def histogram(w):
    w = _u16(w)
    cnt = np.zeros(256, np.uint64)
    lib().nzo_histogram(_p(w, ctypes.c_uint16), w.size, _p(cnt, ctypes.c_uint64))
    return cnt


def entropy(cnt):
    cnt = np.ascontiguousarray(cnt, dtype=np.uint64)
    return float(lib().nzo_entropy(_p(cnt, ctypes.c_uint64)))


def cross_entropy(cnt, freq):
    cnt = np.ascontiguousarray(cnt, dtype=np.uint64)
    freq = np.ascontiguousarray(freq, dtype=np.uint16)
    return float(lib().nzo_cross_entropy(_p(cnt, ctypes.c_uint64), _p(freq, ctypes.c_uint16)))


def quantise(cnt, guard=0):
    cnt = np.ascontiguousarray(cnt, dtype=np.uint64)
    freq = np.zeros(256, np.uint16)
    if guard:
        rc = lib().nzo_quantise_guarded(_p(cnt, ctypes.c_uint64), guard, _p(freq, ctypes.c_uint16))
    else:
        rc = lib().nzo_quantise(_p(cnt, ctypes.c_uint64), _p(freq, ctypes.c_uint16))
    if rc != OK:
        raise OracleError(rc, "quantise")
    return freq


def rans_encode_step(x, f, c):
    """One encoder step -> (new state, emitted word or None)."""
    word, emitted = ctypes.c_uint16(0), ctypes.c_int(0)
    xn = lib().nzo_rans_encode_step(x, f, c, ctypes.byref(word), ctypes.byref(emitted))
    return int(xn), (int(word.value) if emitted.value else None)


def rans_decode_step(x, f, c, next_word=0):
    """One decoder step for a state whose slot lies in [c, c+f) -> (new state, word consumed?)."""
    consumed = ctypes.c_int(0)
    xn = lib().nzo_rans_decode_step(x, f, c, next_word, ctypes.byref(consumed))
    return int(xn), bool(consumed.value)


def encode_chunk(sym, freq, k_states=K, g=G, words_cap=None):
    """Returns (states[K] u32, lens[K] u16, list of K word arrays)."""
    sym = np.ascontiguousarray(sym, dtype=np.uint8)
    freq = np.ascontiguousarray(freq, dtype=np.uint16)
    if words_cap is None:
        words_cap = max(1, sym.size)
    states = np.zeros(k_states, np.uint32)
    lens = np.zeros(k_states, np.uint16)
    words = np.zeros(k_states * words_cap, np.uint16)
    rc = lib().nzo_encode_chunk(_p(sym, ctypes.c_uint8), sym.size, _p(freq, ctypes.c_uint16),
                                k_states, g, _p(states, ctypes.c_uint32), _p(lens, ctypes.c_uint16),
                                _p(words, ctypes.c_uint16), words_cap)
    if rc != OK:
        raise OracleError(rc, "encode_chunk")
    runs = [words[j * words_cap: j * words_cap + int(lens[j])].copy() for j in range(k_states)]
    return states, lens, runs


def decode_chunk(m, freq, states, runs, k_states=K, g=G):
    freq = np.ascontiguousarray(freq, dtype=np.uint16)
    states = np.ascontiguousarray(states, dtype=np.uint32)
    words_cap = max([1] + [len(r) for r in runs])
    lens = np.array([len(r) for r in runs], np.uint16)
    words = np.zeros(k_states * words_cap, np.uint16)
    for j, r in enumerate(runs):
        words[j * words_cap: j * words_cap + len(r)] = r
    sym = np.zeros(m, np.uint8)
    rc = lib().nzo_decode_chunk(_p(sym, ctypes.c_uint8), m, _p(freq, ctypes.c_uint16), k_states, g,
                                _p(states, ctypes.c_uint32), _p(lens, ctypes.c_uint16),
                                _p(words, ctypes.c_uint16), words_cap)
    if rc != OK:
        raise OracleError(rc, "decode_chunk")
    return sym


def block_coefficients(w, block):
    w = _u16(w)
    coef = np.zeros(int(lib().nzo_block_count(w.size, block)), np.uint8)
    rc = lib().nzo_block_coefficients(_p(w, ctypes.c_uint16), w.size, block, _p(coef, ctypes.c_uint8))
    if rc != OK:
        raise OracleError(rc, "block_coefficients")
    return coef


def normalise(w, block, coef):
    w = _u16(w)
    coef = np.ascontiguousarray(coef, dtype=np.uint8)
    out = np.empty_like(w)
    lib().nzo_normalise(_p(w, ctypes.c_uint16), w.size, block, _p(coef, ctypes.c_uint8), _p(out, ctypes.c_uint16))
    return out


def denormalise(w, block, coef):
    w = _u16(w)
    coef = np.ascontiguousarray(coef, dtype=np.uint8)
    out = np.empty_like(w)
    lib().nzo_denormalise(_p(w, ctypes.c_uint16), w.size, block, _p(coef, ctypes.c_uint8), _p(out, ctypes.c_uint16))
    return out


def lossy_blockwise(w, k, block):
    """What decompress(compress_blockwise(w)) must return, from the three steps alone."""
    coef = block_coefficients(w, block)
    return denormalise(truncate(normalise(w, block, coef), k), block, coef)


def compress(w, k=7, threads=1, block=0, guard=0, freq=None):
    """bf16 words (uint16 array) -> container bytes (uint8 array).

    guard: the table keeps f >= 1 that far beyond the occupied exponents; freq: code with this
    earlier table instead of fresh statistics (OracleError with code ESTALE if it cannot)."""
    w = _u16(w)
    cap = int(lib().nzo_compress_bound(w.size, k if k in (7, 3, 1, 0) else 7))
    blob = np.empty(cap, np.uint8)
    written = ctypes.c_uint64(0)
    if freq is not None:
        if block:
            raise ValueError("an earlier table cannot be combined with block-wise normalisation")
        freq = np.ascontiguousarray(freq, dtype=np.uint16)
        rc = lib().nzo_compress_with_table(_p(w, ctypes.c_uint16), w.size, k, _p(freq, ctypes.c_uint16), guard,
                                           _p(blob, ctypes.c_uint8), cap, ctypes.byref(written), threads)
    elif guard:
        if block:
            raise ValueError("a guard band cannot be combined with block-wise normalisation")
        rc = lib().nzo_compress_guarded(_p(w, ctypes.c_uint16), w.size, k, guard, _p(blob, ctypes.c_uint8), cap,
                                        ctypes.byref(written), threads)
    elif block:
        rc = lib().nzo_compress_blockwise(_p(w, ctypes.c_uint16), w.size, k, block, _p(blob, ctypes.c_uint8), cap,
                                          ctypes.byref(written), threads)
    else:
        rc = lib().nzo_compress(_p(w, ctypes.c_uint16), w.size, k, _p(blob, ctypes.c_uint8), cap,
                                ctypes.byref(written), threads)
    if rc != OK:
        raise OracleError(rc, "compress")
    return blob[: written.value].copy()


def decompress(blob, n, threads=1):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    out = np.empty(n, np.uint16)
    rc = lib().nzo_decompress(_p(blob, ctypes.c_uint8), blob.size, _p(out, ctypes.c_uint16), n, threads)
    if rc != OK:
        raise OracleError(rc, "decompress")
    return out


def compress_f32(w, threads=1, guard=0, freq=None):
    """binary32 words (uint32 array) -> container bytes: upper halves through the lossless bf16 path,
    lower halves as a raw plane.  guard / freq as in compress()."""
    w = np.ascontiguousarray(w)
    if w.dtype != np.uint32:
        raise TypeError("binary32 words must be passed as uint32")
    w = w.reshape(-1)
    cap = int(lib().nzo_compress_bound(w.size, 7))
    blob = np.empty(cap, np.uint8)
    written = ctypes.c_uint64(0)
    table = None
    if freq is not None:
        table = np.ascontiguousarray(freq, dtype=np.uint16)
        if table.size != 256:
            raise ValueError("a frequency table has 256 entries")
    rc = lib().nzo_compress_f32_with_table(_p(w, ctypes.c_uint32), w.size,
                                           None if table is None else _p(table, ctypes.c_uint16), guard,
                                           _p(blob, ctypes.c_uint8), cap, ctypes.byref(written), threads)
    if rc != OK:
        raise OracleError(rc, "compress_f32")
    return blob[: written.value].copy()


def decompress_f32(blob, n, threads=1):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    out = np.empty(n, np.uint32)
    rc = lib().nzo_decompress_f32(_p(blob, ctypes.c_uint8), blob.size, _p(out, ctypes.c_uint32), n, threads)
    if rc != OK:
        raise OracleError(rc, "decompress_f32")
    return out


def compress_f16(w, threads=1, guard=0, freq=None):
    """binary16 words (uint16 array) -> container bytes: the upper byte of a word is the coded symbol,
    the lower byte is stored raw.  guard / freq as in compress()."""
    w = np.ascontiguousarray(w)
    if w.dtype != np.uint16:
        raise TypeError("binary16 words must be passed as uint16")
    w = w.reshape(-1)
    cap = int(lib().nzo_compress_bound(w.size, 7))
    blob = np.empty(cap, np.uint8)
    written = ctypes.c_uint64(0)
    table = None
    if freq is not None:
        table = np.ascontiguousarray(freq, dtype=np.uint16)
        if table.size != 256:
            raise ValueError("a frequency table has 256 entries")
    rc = lib().nzo_compress_f16(_p(w, ctypes.c_uint16), w.size, None if table is None else _p(table, ctypes.c_uint16),
                                guard, _p(blob, ctypes.c_uint8), cap, ctypes.byref(written), threads)
    if rc != OK:
        raise OracleError(rc, "compress_f16")
    return blob[: written.value].copy()


def decompress_f16(blob, n, threads=1):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    out = np.empty(n, np.uint16)
    rc = lib().nzo_decompress_f16(_p(blob, ctypes.c_uint8), blob.size, _p(out, ctypes.c_uint16), n, threads)
    if rc != OK:
        raise OracleError(rc, "decompress_f16")
    return out


def blob_info(blob):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    n, k, tw = ctypes.c_uint64(0), ctypes.c_int(0), ctypes.c_uint64(0)
    freq = np.zeros(256, np.uint16)
    rc = lib().nzo_blob_info(_p(blob, ctypes.c_uint8), blob.size, ctypes.byref(n), ctypes.byref(k),
                             ctypes.byref(tw), _p(freq, ctypes.c_uint16))
    if rc != OK:
        raise OracleError(rc, "blob_info")
    return {"n": n.value, "k": k.value, "total_words": tw.value, "freq": freq}


def sections(blob):
    """Byte ranges of the container's sections, for tests that compare them one by one."""
    info = blob_info(blob)
    n, k, tw = info["n"], info["k"], info["total_words"]
    block = int(np.ascontiguousarray(blob[48:52]).view("<u4")[0])
    f32 = int(np.ascontiguousarray(blob[56:60]).view("<u4")[0]) == 1
    nc = (n + CHUNK - 1) // CHUNK
    pad = lambda v: (v + 15) & ~15
    out, pos = {}, 0
    for name, size in (("header", HEADER_BYTES), ("freq", 512), ("offsets", pad((nc + 1) * 4)),
                       ("states", nc * K * 4), ("lens", nc * K), ("words", pad(tw * 2)),
                       ("signmant", pad(signmant_bytes(n, k))), ("low", pad(2 * n) if f32 else 0),
                       ("coef", pad((n + block - 1) // block) if block else 0)):
        out[name] = (pos, pos + size)
        pos += size
    return out
