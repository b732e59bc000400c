"""GPU parity for binary16 tensors (-m gpu).

The paper compresses BFloat16 weights (Sec. 2.1).  For IEEE binary16 the library codes the upper
byte of every word (sign, 5 exponent bits, 2 mantissa bits) in place of the bf16 exponent byte and
stores the lower byte raw; the oracle states the container (oracle.compress_f16) and the HIP path
has to produce the same bytes and return the same words.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2410_20650_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def nz():
    from paper_2410_20650_amd import binding
    return binding


def same_container(got, want, what):
    if got.size != want.size or not np.array_equal(got, want):
        sec = O.sections(want)
        bad = [name for name, (lo, hi) in sec.items() if not np.array_equal(got[lo:hi], want[lo:hi])]
        raise AssertionError(f"{what}: container differs from the oracle's in sections {bad} "
                             f"({got.size} vs {want.size} bytes)")


def decoded(nz, blob, like):
    out = torch.full_like(like, float("nan"))
    nz.neuzip_decompress(blob, out)
    nz.neuzip_check(blob)
    return inputs.bits16(out)


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 4095, 4096, 4097, 16 * 4096 + 13, 33 * 4096 + 2049, 1_000_003, 5_000_000])
def test_f16_container_and_round_trip(nz, n):
    w = inputs.gaussian_f16(n, 12_000 + n % 977, device=DEV)
    words = inputs.bits16(w)
    blob = nz.neuzip_compress(w, 7)
    assert blob.dtype == nz.F16 and blob.elems == n and blob.mantissa_bits == 7
    want = O.compress_f16(words, threads=8)
    same_container(nz.neuzip_export(blob), want, f"n={n}")
    if n:
        assert np.array_equal(decoded(nz, blob, w), words)
        assert np.array_equal(nz.neuzip_histogram(blob), np.bincount(words >> 8, minlength=256))
    assert np.array_equal(O.decompress_f16(nz.neuzip_export(blob), n, threads=8), words)
    back = nz.neuzip_import(want)
    assert back.dtype == nz.F16
    if n:
        assert np.array_equal(decoded(nz, back, w), words)


def test_f16_every_pattern_and_extremes(nz):
    w = inputs.all_patterns_f16(device=DEV)
    blob = nz.neuzip_compress(w, 7)
    same_container(nz.neuzip_export(blob), O.compress_f16(inputs.bits16(w)), "all patterns")
    out = torch.zeros_like(w)
    nz.neuzip_decompress(blob, out)
    nz.neuzip_check(blob)
    assert np.array_equal(inputs.bits16(out), inputs.bits16(w))
    # one upper byte only: the decoder's path without words
    c = inputs.from_bits16((0x3A00 + (np.arange(70_001) % 256)).astype(np.uint16), DEV)
    blob = nz.neuzip_compress(c, 7)
    same_container(nz.neuzip_export(blob), O.compress_f16(inputs.bits16(c)), "single symbol")
    assert np.array_equal(decoded(nz, blob, c), inputs.bits16(c))
    # uniformly random words: 8 bits per symbol, the words do not fit the LDS window
    r = inputs.from_bits16(inputs.bits(inputs.random_bits_bf16(300_000, 12_100)), DEV)
    blob = nz.neuzip_compress(r, 7)
    same_container(nz.neuzip_export(blob), O.compress_f16(inputs.bits16(r), threads=8), "random bits")
    assert np.array_equal(decoded(nz, blob, r), inputs.bits16(r))


def test_f16_recompress_batches_and_streaming_size(nz):
    n = 16 * 4096 * 3 + 777
    w0 = inputs.gaussian_f16(n, 12_200, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w0], 7, 4)
    same_container(nz.neuzip_export(blob), O.compress_f16(inputs.bits16(w0), threads=8, guard=4), "guarded")
    table = nz.neuzip_frequencies(blob).copy()
    w = w0
    for step in range(2):
        w = inputs.synthetic_update(w, seed=12_201 + step)
        (rebuilt,) = nz.neuzip_recompress([w], [blob])
        assert rebuilt == 0
        same_container(nz.neuzip_export(blob), O.compress_f16(inputs.bits16(w), threads=8, guard=4, freq=table),
                       f"step {step}")
        assert np.array_equal(decoded(nz, blob, w), inputs.bits16(w))
    words = inputs.bits16(w).copy()
    words[n - 2] = 0xFBFF                                          # an upper byte the table has no room for
    w = inputs.from_bits16(words, DEV)
    (rebuilt,) = nz.neuzip_recompress([w], [blob])
    assert rebuilt == 1
    same_container(nz.neuzip_export(blob), O.compress_f16(words, threads=8, guard=4), "fallback")
    # a layer in one call, then decoded in one launch next to a bf16 blob
    shapes = [(512, 512), (128, 512), (77, 13), (0,), (512, 1792)]
    ws = [inputs.gaussian_f16(s, 12_300 + i, device=DEV) for i, s in enumerate(shapes)]
    blobs = nz.neuzip_compress_batch(ws, 7)
    h = inputs.gaussian_bf16(50_000, 12_310, device=DEV)
    hb = nz.neuzip_compress(h, 7)
    outs = [torch.zeros_like(t) for t in ws] + [torch.zeros_like(h)]
    nz.neuzip_decompress_batch(blobs + [hb], outs)
    for t, b, o in zip(ws, blobs, outs):
        nz.neuzip_check(b)
        same_container(nz.neuzip_export(b), O.compress_f16(inputs.bits16(t), threads=8), str(tuple(t.shape)))
        assert np.array_equal(inputs.bits16(o), inputs.bits16(t))
    assert np.array_equal(inputs.bits(outs[-1]), inputs.bits(h))
    # beyond 2^26 elements the decoder stores non-temporally
    n = (64 << 20) + 4096 + 5
    big = inputs.gaussian_f16(n, 12_400, device=DEV)
    blob = nz.neuzip_compress(big, 7)
    out = torch.zeros_like(big)
    nz.neuzip_decompress(blob, out)
    nz.neuzip_check(blob)
    assert torch.equal(out.view(torch.int16), big.view(torch.int16))
    same_container(nz.neuzip_export(blob), O.compress_f16(inputs.bits16(big), threads=8), "streaming size")


def test_f16_argument_errors(nz):
    w = inputs.gaussian_f16(10_000, 12_500, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    lib = nz.library()
    none = ctypes.c_void_p(None)
    for k in (3, 1, 0):
        handle = ctypes.c_void_p(None)
        assert lib.neuzip_compress(ctypes.c_void_p(w.data_ptr()), w.numel(), nz.F16, k, none,
                                   ctypes.byref(handle)) == nz.EUNSUPPORTED
    # a binary16 blob takes no bf16 tensor and decodes into no bf16 buffer
    h = inputs.gaussian_bf16(10_000, 12_501, device=DEV)
    handle = ctypes.c_void_p(blob.handle.value)
    assert lib.neuzip_compress(ctypes.c_void_p(h.data_ptr()), h.numel(), nz.BF16, 7, none,
                               ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_decompress(blob.handle, ctypes.c_void_p(h.data_ptr()), h.numel(), nz.BF16, none) == nz.EINVAL
    x = inputs.gaussian_bf16((2, 128), 12_502, device=DEV)
    half = nz.neuzip_compress(inputs.gaussian_f16(16 * 128, 12_503, device=DEV), 7)
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_linear(half, 16, 128, x)
    assert err.value.code == nz.EUNSUPPORTED
    assert np.array_equal(decoded(nz, blob, w), inputs.bits16(w))
