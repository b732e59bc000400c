"""GPU parity of the guard-band tables and of recompression with a kept table (-m gpu).

Alg. 1 compresses every weight again after each update.  The oracle states what the container
must be when the table of the step before is reused (oracle.compress(..., freq=...)) and what a
guard-band table is (oracle.quantise(..., guard=...)); the HIP path has to produce the same bytes.
"""
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
    return inputs.bits(out)


@pytest.mark.parametrize("guard", [0, 1, 8, 255])
@pytest.mark.parametrize("n", [1, 4097, 200_000 + 3])
def test_guard_band_table_matches_the_oracle(nz, n, guard):
    w = inputs.gaussian_bf16(n, 8100 + n, device=DEV)
    words = inputs.bits(w)
    (blob,) = nz.neuzip_compress_guarded([w], 7, guard)
    assert blob.guard == guard
    assert np.array_equal(nz.neuzip_frequencies(blob), O.quantise(O.histogram(words), guard=guard))
    same_container(nz.neuzip_export(blob), O.compress(words, 7, threads=8, guard=guard), f"guard {guard}")
    assert np.array_equal(decoded(nz, blob, w), words)
    # the guard survives export and import
    back = nz.neuzip_import(nz.neuzip_export(blob))
    assert back.guard == guard
    assert np.array_equal(decoded(nz, back, w), words)


def test_a_guarded_blob_keeps_its_guard_when_compressed_into_again(nz):
    w0 = inputs.gaussian_bf16(100_000, seed=4100, device=DEV)
    w1 = inputs.gaussian_bf16(100_000, seed=4101, std=0.05, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w0], 7, 8)
    for call in (lambda: nz.neuzip_compress(w1, 7, blob=blob), lambda: nz.neuzip_compress_batch([w1], 7, 0, blobs=[blob]),
                 lambda: nz.neuzip_compress_noalloc(w1, 7, blob)):
        nz.neuzip_compress_guarded([w0], 7, 8, blobs=[blob])
        call()
        assert blob.guard == 8
        same_container(nz.neuzip_export(blob), O.compress(inputs.bits(w1), 7, threads=8, guard=8), "guard kept")
    nz.neuzip_compress_guarded([w1], 7, 0, blobs=[blob])             # the guarded entry point sets it anew
    assert blob.guard == 0
    same_container(nz.neuzip_export(blob), O.compress(inputs.bits(w1), 7, threads=8), "guard dropped")


def test_guard_band_on_every_pattern_and_on_a_single_exponent(nz):
    w = inputs.all_patterns_bf16(device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w], 7, 3)
    same_container(nz.neuzip_export(blob), O.compress(inputs.bits(w), 7, guard=3), "all patterns")
    c = inputs.constant_bf16(10_000, 0.75, device=DEV)       # one exponent: the band makes it 1 + 2*4 symbols, + exponent 0
    (blob,) = nz.neuzip_compress_guarded([c], 7, 4)
    f = nz.neuzip_frequencies(blob)
    assert np.count_nonzero(f) == 10 and f.max() == 4096 - 9 and f[0] == 1
    same_container(nz.neuzip_export(blob), O.compress(inputs.bits(c), 7, guard=4), "single exponent")
    assert np.array_equal(decoded(nz, blob, c), inputs.bits(c))


@pytest.mark.parametrize("k", [7, 3, 1, 0])
@pytest.mark.parametrize("n", [5, 4096, 3 * 4096 + 1001, 33 * 4096 + 5, 1_000_003])
def test_recompress_with_the_kept_table_matches_the_oracle(nz, n, k):
    guard = 8
    w0 = inputs.gaussian_bf16(n, 8200 + n, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w0], k, guard)
    table = nz.neuzip_frequencies(blob).copy()
    w = w0
    for step in range(3):
        w = inputs.synthetic_update(w, seed=8300 + 10 * n + step)
        words = inputs.bits(w)
        covered = bool(np.all(table[O.split(words)[1]] > 0))
        (rebuilt,) = nz.neuzip_recompress([w], [blob])
        if covered:
            assert rebuilt == 0
            want = O.compress(words, k, threads=8, guard=guard, freq=table)
        else:                                                  # the update left the band: fresh statistics
            assert rebuilt == 1
            want = O.compress(words, k, threads=8, guard=guard)
            table = O.blob_info(want)["freq"]
        same_container(nz.neuzip_export(blob), want, f"step {step}")
        assert np.array_equal(decoded(nz, blob, w), O.truncate(words, k))
        assert np.array_equal(nz.neuzip_frequencies(blob), table)
        assert blob.guard == guard and blob.mantissa_bits == k


def test_recompress_falls_back_when_an_exponent_has_no_room(nz):
    n = 70_000
    w0 = inputs.gaussian_bf16(n, 8400, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w0], 7, 1)
    table = nz.neuzip_frequencies(blob).copy()
    top = int(np.nonzero(table)[0][-1])
    words = inputs.bits(w0).copy()
    words[n - 3] = np.uint16((top + 2) << 7)                   # far above the band, in the ragged last chunk
    w = inputs.from_bits(words, DEV)
    with pytest.raises(O.OracleError):
        O.compress(words, 7, guard=1, freq=table)
    (rebuilt,) = nz.neuzip_recompress([w], [blob])
    assert rebuilt == 1
    same_container(nz.neuzip_export(blob), O.compress(words, 7, threads=8, guard=1), "fallback")
    assert np.array_equal(decoded(nz, blob, w), words)
    assert np.array_equal(nz.neuzip_histogram(blob).astype(np.uint64), O.histogram(words))
    # and the new table then serves the next step
    (rebuilt,) = nz.neuzip_recompress([w0], [blob])
    assert rebuilt == 0
    same_container(nz.neuzip_export(blob),
                   O.compress(inputs.bits(w0), 7, threads=8, guard=1, freq=nz.neuzip_frequencies(blob)), "next step")
    assert np.array_equal(decoded(nz, blob, w0), inputs.bits(w0))


def test_recompress_a_layer_in_one_call_with_one_stale_tensor(nz):
    shapes = [(512, 512), (128, 512), (128, 512), (512, 512), (512, 1792), (512, 1792), (1792, 512), (77, 13), (0,)]
    ws = [inputs.gaussian_bf16(s, 8500 + i, device=DEV) for i, s in enumerate(shapes)]
    blobs = nz.neuzip_compress_guarded(ws, 7, 8)
    tables = [nz.neuzip_frequencies(b).copy() for b in blobs]
    new = [inputs.synthetic_update(w, seed=8600 + i) for i, w in enumerate(ws)]
    # tensor 4 gets a value its table cannot code
    words4 = inputs.bits(new[4]).copy()
    words4[12345] = np.uint16((int(np.nonzero(tables[4])[0][-1]) + 1) << 7)
    new[4] = inputs.from_bits(words4, DEV).reshape(shapes[4])
    rebuilt = nz.neuzip_recompress(new, blobs)
    assert rebuilt == [0, 0, 0, 0, 1, 0, 0, 0, 0]
    for i, (w, b) in enumerate(zip(new, blobs)):
        words = inputs.bits(w)
        want = (O.compress(words, 7, guard=8) if rebuilt[i]
                else O.compress(words, 7, guard=8, freq=tables[i]))
        same_container(nz.neuzip_export(b), want, f"tensor {i}")
        if w.numel():
            assert np.array_equal(decoded(nz, b, w.reshape(-1)), words)


def test_recompress_of_imported_and_of_normalised_blobs(nz):
    n = 50_000
    w0 = inputs.gaussian_bf16(n, 8700, device=DEV)
    w1 = inputs.synthetic_update(w0, seed=8701)
    # a container written by the oracle, imported, then recompressed with its table
    first = O.compress(inputs.bits(w0), 7, guard=8)
    blob = nz.neuzip_import(first)
    (rebuilt,) = nz.neuzip_recompress([w1], [blob])
    assert rebuilt == 0
    same_container(nz.neuzip_export(blob),
                   O.compress(inputs.bits(w1), 7, guard=8, freq=O.blob_info(first)["freq"]), "imported")
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_histogram(blob)                              # no counts were taken
    # block-wise normalised blobs need the block maxima first: always the two-pass route
    lossy = nz.neuzip_compress_blockwise(w0, 3, 128)
    (rebuilt,) = nz.neuzip_recompress([w1], [lossy])
    assert rebuilt == 1
    same_container(nz.neuzip_export(lossy), O.compress(inputs.bits(w1), 3, block=128), "normalised")
    assert np.array_equal(decoded(nz, lossy, w1), O.lossy_blockwise(inputs.bits(w1), 3, 128))


def test_recompress_argument_errors(nz):
    w = inputs.gaussian_bf16(5000, 8800, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w], 7, 2)
    with pytest.raises(ValueError):
        nz.neuzip_recompress([w[:100].contiguous()], [blob])
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_recompress([w, w], [blob, blob])             # one blob cannot receive two tensors
    assert err.value.code == nz.EINVAL
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_compress_guarded([w], 7, 256)
    assert np.array_equal(decoded(nz, blob, w), inputs.bits(w))   # untouched by the failed calls
