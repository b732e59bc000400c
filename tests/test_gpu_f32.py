"""GPU parity for binary32 tensors (-m gpu).

The paper compresses BFloat16 weights (Sec. 2.1).  A binary32 word has the same sign and exponent
bits in its upper half, so the library sends that half through the lossless path unchanged and
keeps the lower half as a raw plane; the oracle states the resulting container
(oracle.compress_f32) and the HIP path has to produce the same bytes and return the same words.
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
    return inputs.bits32(out)


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 4095, 4096, 4097, 16 * 4096 + 13, 33 * 4096 + 2049, 1_000_003, 5_000_000])
def test_f32_container_and_round_trip(nz, n):
    w = inputs.gaussian_f32(n, 9800 + n % 977, device=DEV)
    words = inputs.bits32(w)
    blob = nz.neuzip_compress(w, 7)
    assert blob.dtype == nz.F32 and blob.elems == n and blob.mantissa_bits == 7
    want = O.compress_f32(words, threads=8)
    same_container(nz.neuzip_export(blob), want, f"n={n}")
    assert blob.compressed_bytes == want.size
    if n:
        assert np.array_equal(decoded(nz, blob, w), words)
        assert np.array_equal(nz.neuzip_histogram(blob).astype(np.uint64),
                              O.histogram((words >> 16).astype(np.uint16)))
    # the oracle decodes what the GPU wrote, the GPU decodes what the oracle wrote
    assert np.array_equal(O.decompress_f32(nz.neuzip_export(blob), n, threads=8), words)
    back = nz.neuzip_import(want)
    assert back.dtype == nz.F32
    if n:
        assert np.array_equal(decoded(nz, back, w), words)


@pytest.mark.parametrize("low", [0, 1, 0x8000, 0xFFFF, 0x1234])
def test_f32_every_upper_half(nz, low):
    # zeros, subnormals, infinities and NaN payloads of either sign: bit patterns travel untouched
    w = inputs.all_upper_halves_f32(low, device=DEV)
    words = inputs.bits32(w)
    blob = nz.neuzip_compress(w, 7)
    same_container(nz.neuzip_export(blob), O.compress_f32(words, threads=8), f"low={low:#x}")
    out = torch.zeros_like(w)
    nz.neuzip_decompress(blob, out)
    nz.neuzip_check(blob)
    assert np.array_equal(inputs.bits32(out), words)


def test_f32_single_exponent_and_wide_spread(nz):
    c = torch.full((70_001,), 0.75, dtype=torch.float32, device=DEV) + \
        torch.arange(70_001, device=DEV, dtype=torch.float32) * 2.0 ** -24   # one exponent, busy lower halves
    words = inputs.bits32(c)
    assert np.unique(words >> 23).size == 1
    blob = nz.neuzip_compress(c, 7)
    same_container(nz.neuzip_export(blob), O.compress_f32(words), "single exponent")
    assert np.array_equal(decoded(nz, blob, c), words)
    # random 32-bit patterns: over 5 bits per exponent, the decoder reads the words from the blob
    g = torch.Generator(device=DEV).manual_seed(9811)
    v = torch.randint(-2 ** 31, 2 ** 31, (300_000,), generator=g, device=DEV, dtype=torch.int64)
    w = v.to(torch.int32).view(torch.float32)
    words = inputs.bits32(w)
    blob = nz.neuzip_compress(w, 7)
    same_container(nz.neuzip_export(blob), O.compress_f32(words, threads=8), "random bits")
    assert np.array_equal(decoded(nz, blob, w), words)


def test_f32_recompress_with_the_kept_table(nz):
    n = 16 * 4096 * 3 + 777
    w0 = inputs.gaussian_f32(n, 9820, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w0], 7, 8)
    assert blob.guard == 8 and blob.dtype == nz.F32
    same_container(nz.neuzip_export(blob), O.compress_f32(inputs.bits32(w0), threads=8, guard=8), "guarded")
    table = nz.neuzip_frequencies(blob).copy()
    w = w0
    for step in range(3):
        w = inputs.synthetic_update(w, seed=9821 + step)
        words = inputs.bits32(w)
        (rebuilt,) = nz.neuzip_recompress([w], [blob])
        assert rebuilt == 0
        same_container(nz.neuzip_export(blob), O.compress_f32(words, threads=8, guard=8, freq=table), f"step {step}")
        assert np.array_equal(decoded(nz, blob, w), words)
    # a value outside the band: fresh statistics
    words = inputs.bits32(w).copy()
    words[n - 2] = np.uint32((int(np.nonzero(table)[0][-1]) + 12) << 23) | np.uint32(0x4321)
    w = inputs.from_bits32(words, DEV)
    (rebuilt,) = nz.neuzip_recompress([w], [blob])
    assert rebuilt == 1
    same_container(nz.neuzip_export(blob), O.compress_f32(words, threads=8, guard=8), "fallback")
    assert np.array_equal(decoded(nz, blob, w), words)


def test_f32_batches_and_sequence(nz):
    shapes = [(512, 512), (128, 512), (77, 13), (0,), (512, 1792), (3, 4096)]
    ws = [inputs.gaussian_f32(s, 9830 + i, device=DEV) for i, s in enumerate(shapes)]
    blobs = nz.neuzip_compress_batch(ws, 7)
    for w, b in zip(ws, blobs):
        same_container(nz.neuzip_export(b), O.compress_f32(inputs.bits32(w), threads=8), str(tuple(w.shape)))
    # a batch that mixes binary32 and bf16 blobs: each kind gets its own launches
    h = inputs.gaussian_bf16(50_000, 9840, device=DEV)
    hb = nz.neuzip_compress(h, 7)
    outs = [torch.zeros_like(w) for w in ws] + [torch.zeros_like(h)]
    nz.neuzip_decompress_batch(blobs + [hb], outs)
    for b in blobs + [hb]:
        nz.neuzip_check(b)
    for w, o in zip(ws, outs):
        assert np.array_equal(inputs.bits32(o), inputs.bits32(w))
    assert np.array_equal(inputs.bits(outs[-1]), inputs.bits(h))
    # one scratch buffer for all, sized for the largest tensor in 16-bit words
    scratch = torch.zeros(512 * 1792, dtype=torch.float32, device=DEV)
    at = nz.neuzip_decompress_sequence(blobs + [hb], scratch)
    torch.cuda.synchronize()
    assert at[-1] == 0                                   # another element type: a group of its own
    assert np.array_equal(inputs.bits(scratch.view(torch.bfloat16)[:50_000]), inputs.bits(h))
    at = nz.neuzip_decompress_sequence(blobs, scratch)
    assert np.array_equal(inputs.bits32(scratch[at[-1]: at[-1] + 3 * 4096]), inputs.bits32(ws[-1]))
    small = torch.zeros(512 * 1792 - 8, dtype=torch.float32, device=DEV)
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_decompress_sequence(blobs, small)


def test_f32_argument_errors(nz):
    w = inputs.gaussian_f32(10_000, 9850, device=DEV)
    h = inputs.gaussian_bf16(10_000, 9851, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    lib = nz.library()
    none = ctypes.c_void_p(None)
    for k in (3, 1, 0):                                             # lossless only
        handle = ctypes.c_void_p(None)
        assert lib.neuzip_compress(ctypes.c_void_p(w.data_ptr()), w.numel(), nz.F32, k, none,
                                   ctypes.byref(handle)) == nz.EUNSUPPORTED
    handle = ctypes.c_void_p(None)
    assert lib.neuzip_compress(ctypes.c_void_p(w.data_ptr()), w.numel(), 3, 7, none, ctypes.byref(handle)) == nz.EINVAL
    # element types do not mix: a binary32 blob takes no bf16 tensor and decodes into no bf16 buffer
    handle = ctypes.c_void_p(blob.handle.value)
    assert lib.neuzip_compress(ctypes.c_void_p(h.data_ptr()), h.numel(), nz.BF16, 7, none,
                               ctypes.byref(handle)) == nz.EINVAL
    assert lib.neuzip_decompress(blob.handle, ctypes.c_void_p(w.data_ptr()), w.numel(), nz.BF16, none) == nz.EINVAL
    hb = nz.neuzip_compress(h, 7)
    assert lib.neuzip_decompress(hb.handle, ctypes.c_void_p(w.data_ptr()), h.numel(), nz.F32, none) == nz.EINVAL
    x = inputs.gaussian_bf16((2, 128), 9852, device=DEV)
    wide = nz.neuzip_compress(inputs.gaussian_f32(16 * 128, 9853, device=DEV), 7)
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_linear(wide, 16, 128, x)
    assert err.value.code == nz.EUNSUPPORTED
    # a container whose element-type word is damaged is refused
    c = nz.neuzip_export(blob).copy()
    c[56] = 2
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_import(c)
    c[56] = 0                                                       # now the size no longer fits
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_import(c)
    assert np.array_equal(decoded(nz, blob, w), inputs.bits32(w))   # untouched by the failed calls


def test_f32_tensor_that_streams_to_hbm(nz):
    # from 2^25 elements on the decoder stores non-temporally and the lanes of an octet trade
    # 16-byte pieces so that every store instruction covers whole cache lines
    n = (32 << 20) + 4096 + 1234
    w = inputs.gaussian_f32(n, 9860, device=DEV)
    words = inputs.bits32(w)
    blob = nz.neuzip_compress(w, 7)
    out = torch.zeros_like(w)
    nz.neuzip_decompress(blob, out)
    nz.neuzip_check(blob)
    assert np.array_equal(inputs.bits32(out), words)
    same_container(nz.neuzip_export(blob), O.compress_f32(words, threads=8), "streaming size")
    # the same decoder inside a batch, next to a small tensor and a bf16 one
    small = inputs.gaussian_f32(70_000, 9861, device=DEV)
    half = inputs.gaussian_bf16(90_000, 9862, device=DEV)
    blobs = [blob, nz.neuzip_compress(small, 7), nz.neuzip_compress(half, 7)]
    outs = [torch.zeros_like(w), torch.zeros_like(small), torch.zeros_like(half)]
    nz.neuzip_decompress_batch(blobs, outs)
    for b in blobs:
        nz.neuzip_check(b)
    assert np.array_equal(inputs.bits32(outs[0]), words)
    assert np.array_equal(inputs.bits32(outs[1]), inputs.bits32(small))
    assert np.array_equal(inputs.bits(outs[2]), inputs.bits(half))
