"""The entry point that allocates nothing (neuzip_compress_noalloc) against neuzip_compress:
same container byte for byte, same decoded words, on two calls in a row (the second with a smaller
tensor), and its refusals."""
import numpy as np
import pytest
import torch

from paper_2410_20650_amd import inputs

pytestmark = pytest.mark.gpu

MAX_ELEMS = 1 << 22


@pytest.fixture(scope="module")
def nz():
    from paper_2410_20650_amd import binding
    return binding


def roomy_blob(nz, n, k, dtype=torch.bfloat16):
    """A blob of n elements whose word section has room for any stream: made from random bit patterns."""
    seed = inputs.seed_for(13, 100 + n % 1000 + k)
    if dtype == torch.float32:
        noise = inputs.random_bits_bf16(2 * n, seed, device="cuda:0").view(torch.float32)
    else:
        noise = inputs.random_bits_bf16(n, seed, device="cuda:0").view(dtype)
    return nz.neuzip_compress(noise, k)


def check_against_allocating_call(nz, w, k):
    want = nz.neuzip_compress(w, k)
    blob = roomy_blob(nz, w.numel(), k, w.dtype)
    held = blob.device_bytes
    nz.neuzip_compress_noalloc(w, k, blob)
    assert blob.device_bytes == held
    assert np.array_equal(nz.neuzip_export(blob), nz.neuzip_export(want))
    assert np.array_equal(nz.neuzip_histogram(blob), nz.neuzip_histogram(want))
    a, b = torch.empty_like(w), torch.empty_like(w)
    nz.neuzip_decompress(blob, a)
    nz.neuzip_decompress(want, b)
    nz.neuzip_check(blob)
    torch.cuda.synchronize()
    assert torch.equal(a.view(-1).view(torch.uint8), b.view(-1).view(torch.uint8))
    return blob


def test_two_calls_in_a_row_the_second_smaller(nz):
    big = inputs.gaussian_bf16((1024, 4096 - 3), inputs.seed_for(13, 1), device="cuda:0")   # ragged, 1023 + chunks
    small = inputs.gaussian_bf16((300, 1000 + 1), inputs.seed_for(13, 2), device="cuda:0")
    check_against_allocating_call(nz, big, 7)
    check_against_allocating_call(nz, small, 7)
    # and the same blob again, after the workspace has served another tensor in between
    blob = check_against_allocating_call(nz, small, 3)
    check_against_allocating_call(nz, big, 0)
    again = inputs.student_t4_bf16((300, 1000 + 1), inputs.seed_for(13, 3), device="cuda:0")
    want = nz.neuzip_compress(again, 3)
    nz.neuzip_compress_noalloc(again, 3, blob)
    assert np.array_equal(nz.neuzip_export(blob), nz.neuzip_export(want))


def test_other_element_types_and_the_largest_size(nz):
    w32 = inputs.gaussian_f32((512, 1024 + 5), inputs.seed_for(13, 4), device="cuda:0")
    check_against_allocating_call(nz, w32, 7)
    w16 = inputs.gaussian_f16((512, 1024 + 5), inputs.seed_for(13, 5), device="cuda:0")
    check_against_allocating_call(nz, w16, 7)
    full = inputs.gaussian_bf16(MAX_ELEMS, inputs.seed_for(13, 6), device="cuda:0")
    check_against_allocating_call(nz, full, 7)
    empty = torch.empty(0, dtype=torch.bfloat16, device="cuda:0")
    blob = nz.neuzip_compress(empty, 7)
    nz.neuzip_compress_noalloc(empty, 7, blob)
    assert np.array_equal(nz.neuzip_export(blob), nz.neuzip_export(nz.neuzip_compress(empty, 7)))


def test_refusals(nz):
    w = inputs.gaussian_bf16(MAX_ELEMS + 4096, inputs.seed_for(13, 7), device="cuda:0")
    blob = nz.neuzip_compress(w, 7)
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_compress_noalloc(w, 7, blob)                      # beyond the stated maximum
    assert err.value.code == nz.EUNSUPPORTED
    out = torch.empty_like(w)
    nz.neuzip_decompress(blob, out)                                 # untouched by the refused call
    assert torch.equal(out.view(torch.int16), w.view(torch.int16))
    small = w[:8192].contiguous()
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_compress_noalloc(small, 7, blob)                  # size mismatch
    assert err.value.code == nz.EINVAL
    b3 = nz.neuzip_compress(small, 3)
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_compress_noalloc(small, 7, b3)                    # width mismatch
    assert err.value.code == nz.EINVAL
    bn = nz.neuzip_compress_blockwise(small, 3, 64)
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_compress_noalloc(small, 3, bn)                    # normalised blobs are not taken
    assert err.value.code == nz.EUNSUPPORTED
    # a stream longer than the room the blob has: refused, and the blob then holds no tensor
    calm = torch.full((8192,), 0.5, dtype=torch.bfloat16, device="cuda:0")
    tight = nz.neuzip_compress(calm, 7)
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_compress_noalloc(roomy_source(small), 7, tight)
    assert err.value.code == nz.ENOMEM
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_decompress(tight, torch.empty_like(calm))
    nz.neuzip_compress(calm, 7, blob=tight)                         # an allocating call makes it whole again
    nz.neuzip_decompress(tight, out[:8192])
    assert torch.equal(out[:8192].view(torch.int16), calm.view(torch.int16))


def roomy_source(like):
    return inputs.random_bits_bf16(like.numel(), inputs.seed_for(13, 8), device="cuda:0")
