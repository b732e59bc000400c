"""Host-side checks that need no GPU: the C-ABI library loads, exports what the header declares,
and rejects bad arguments and malformed containers before any device work."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import oracle as O
from paper_2410_20650_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nz():
    from paper_2410_20650_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "neuzip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(neuzip_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(nz):
    names = declared_functions()
    assert "neuzip_compress" in names and "neuzip_decompress" in names and "neuzip_free" in names
    lib = nz.library()
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in include/neuzip.h but not exported"
    assert sorted(nz.EXPORTED) == names


def test_binding_mirrors_the_header(nz):
    for name in declared_functions():
        if name in ("neuzip_strerror", "neuzip_last_hip_error", "neuzip_elems", "neuzip_mantissa_bits",
                    "neuzip_device_bytes", "neuzip_block_size", "neuzip_guard", "neuzip_dtype"):
            continue  # surfaced as Blob properties / NeuzipError fields
        assert hasattr(nz, name), f"binding lacks {name}"


def test_error_strings_and_null_handles(nz):
    lib = nz.library()
    for code in (0, -1, -2, -3, -4, -5):
        assert lib.neuzip_strerror(code)
    assert lib.neuzip_strerror(-99) == b"unknown error"
    assert lib.neuzip_compressed_bytes(None) == 0
    assert lib.neuzip_device_bytes(None) == 0
    assert lib.neuzip_elems(None) == 0
    assert lib.neuzip_mantissa_bits(None) == -1
    lib.neuzip_free(None)  # no-op


def test_argument_validation_happens_before_device_work(nz):
    lib = nz.library()
    handle = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)
    # null out-pointer, bad dtype, bad mantissa_bits, misaligned source, oversize
    assert lib.neuzip_compress(fake, 16, 0, 7, None, None) == nz.EINVAL
    assert lib.neuzip_compress(fake, 16, 3, 7, None, ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_compress(fake, 16, nz.F16, 0, None, ctypes.byref(handle)) == nz.EUNSUPPORTED
    assert lib.neuzip_compress(fake, 16, nz.F32, 3, None, ctypes.byref(handle)) == nz.EUNSUPPORTED   # lossless only
    assert lib.neuzip_compress_blockwise(fake, 16, nz.F32, 3, 64, None, ctypes.byref(handle)) == nz.EUNSUPPORTED
    for k in (-1, 2, 4, 5, 6, 8):
        assert lib.neuzip_compress(fake, 16, 0, k, None, ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_compress(ctypes.c_void_p(0x1002), 16, 0, 7, None, ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_compress(None, 16, 0, 7, None, ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_compress(fake, 1 << 32, 0, 7, None, ctypes.byref(handle)) == nz.EUNSUPPORTED
    # block-wise normalisation: only the lossy widths, only the listed block sizes
    assert lib.neuzip_compress_blockwise(fake, 16, 0, 7, 512, None, ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_compress_blockwise(fake, 16, 0, 3, 100, None, ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_compress_blockwise(fake, 16, 0, 3, 16, None, ctypes.byref(handle)) == nz.EINVAL
    assert handle.value is None
    # calls on something that is not a blob
    junk = (ctypes.c_uint8 * 256)()
    assert lib.neuzip_decompress(ctypes.cast(junk, ctypes.c_void_p), fake, 16, 0, None) == nz.EINVAL
    assert lib.neuzip_decompress(None, fake, 16, 0, None) == nz.EINVAL
    assert lib.neuzip_check(None, None) == nz.EINVAL
    assert lib.neuzip_export(None, None, 0, None, None) == nz.EINVAL
    assert lib.neuzip_decompress_sequence(None, 3, fake, 16, None, None) == nz.EINVAL
    assert lib.neuzip_decompress_batch(None, None, 2, None) == nz.EINVAL
    assert lib.neuzip_compress_batch(None, None, 2, 0, 7, 0, None, None) == nz.EINVAL
    assert lib.neuzip_compress_batch(None, None, 0, 0, 7, 0, None, None) == nz.OK
    # guard band and recompression
    assert lib.neuzip_compress_guarded(None, None, 2, 0, 7, 4, None, None) == nz.EINVAL
    srcs = (ctypes.c_void_p * 1)(0x1000)
    sizes = (ctypes.c_uint64 * 1)(16)
    handles = (ctypes.c_void_p * 1)(None)
    assert lib.neuzip_compress_guarded(srcs, sizes, 1, 0, 7, 256, None, handles) == nz.EINVAL
    assert lib.neuzip_recompress(None, 0, None, None, None) == nz.OK
    assert lib.neuzip_recompress(None, 1, None, None, None) == nz.EINVAL
    assert lib.neuzip_recompress(srcs, 1, None, handles, None) == nz.EINVAL      # not a blob
    assert lib.neuzip_guard(None) == 0


def test_import_validates_containers_on_the_host(nz):
    lib = nz.library()
    handle = ctypes.c_void_p(None)

    def try_import(buf):
        buf = np.ascontiguousarray(buf, dtype=np.uint8)
        return lib.neuzip_import(buf.ctypes.data_as(ctypes.c_void_p), buf.size, None, ctypes.byref(handle))

    w = inputs.bits(inputs.gaussian_bf16(20_000, 8))
    good = O.compress(w, 7)
    sec = O.sections(good)
    assert try_import(good[:100]) == nz.ECORRUPT                      # too short
    assert try_import(good[:-16]) == nz.ECORRUPT                      # size does not match the header
    for name, delta, flip in (("header", 0, 1), ("header", 16, 2), ("header", 20, 1), ("header", 28, 1),
                              ("header", 36, 1), ("header", 40, 1), ("freq", 0, 0x10), ("offsets", 4, 1),
                              ("offsets", 20, 0x40), ("lens", 5, 0x80)):
        bad = good.copy()
        bad[sec[name][0] + delta] ^= flip
        assert try_import(bad) == nz.ECORRUPT, (name, delta)
    # a guard band beyond the byte range
    bad = good.copy()
    bad[sec["header"][0] + 53] = 1
    assert try_import(bad) == nz.ECORRUPT
    # a run longer than any state can produce
    bad = good.copy()
    bad[sec["lens"][0]] = 255
    assert try_import(bad) == nz.ECORRUPT
    assert handle.value is None
    assert lib.neuzip_import(None, 100, None, ctypes.byref(handle)) == nz.EINVAL


def test_float_reciprocal_division_scheme_of_the_encoder():
    """The HIP encoder divides the state by a frequency with fp32: q' = trunc(float(x) * rcp) with
    rcp = fl(fl(1/f) * (1 - 2^-21)), then q = q' + (x - q' f >= f).  Emulated here with numpy's IEEE
    fp32 on every frequency and on the dividends that matter (multiples of f and their neighbours,
    the renormalisation limit, random draws): it must equal integer division whenever x < f * 2^20."""
    rng = np.random.default_rng(0)
    one_minus = np.float32(1.0) - np.float32(2.0 ** -21)
    for f in range(1, 4097):
        rcp = np.float32(np.float32(1.0) / np.float32(f)) * one_minus
        limit = min(f << 20, 1 << 32)
        q_edge = np.concatenate([rng.integers(16, 1 << 20, 40), [16, (1 << 20) - 1, (1 << 20) - 2]])
        xs = np.concatenate([q_edge * f, q_edge * f + f - 1, q_edge * f - 1, q_edge * f + 1,
                             rng.integers(1 << 16, limit, 60), [limit - 1, 1 << 16]]).astype(np.int64)
        xs = xs[(xs >= 0) & (xs < limit)]
        est = (xs.astype(np.uint32).astype(np.float32) * rcp).astype(np.int64)     # astype truncates
        rem = xs - est * f
        assert np.all((rem >= 0) & (rem < 2 * f)), f
        q = est + (rem >= f)
        assert np.array_equal(q, xs // f), f
