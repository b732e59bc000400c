"""GPU parity of the weight update of the backward loop (-m gpu).

Alg. 1, backward loop: W_hat <- decompress(c); W_hat <- W_hat - lr * grad; c <- compress(W_hat).
oracle/update.py states the arithmetic of the step (binary32 product and difference, nearest-even
bf16) and the container that results (the kept-table rules of recompression); the HIP path has to
produce the same words and the same bytes.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import oracle as O
from oracle import update as U
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


def one_step(nz, blob, container, g, lr, what, ready=0):
    """Runs the step on the GPU and in the oracle; returns the oracle's new container.  ready = 1, 2:
    the caller decompresses the weight itself and hands it over, as the backward pass does; with 2
    the new weight is not written back."""
    want_container, want_rebuilt, want_words = U.training_step(container, inputs.bits(g), lr, threads=8)
    old_words = O.decompress(container, g.numel(), threads=8)
    space = torch.full_like(g, float("nan"))
    if ready in (1, 2):
        nz.neuzip_decompress(blob, space)
    (rebuilt,) = nz.neuzip_update([blob], [g], [space], lr, weights_ready=ready)
    assert rebuilt == want_rebuilt, what
    if ready >= 2 and not rebuilt:
        assert np.array_equal(inputs.bits(space), old_words), f"{what}: the buffer was to be left alone"
    else:
        assert np.array_equal(inputs.bits(space), want_words), f"{what}: new weights"
    same_container(nz.neuzip_export(blob), want_container, what)
    out = torch.full_like(g, float("nan"))
    nz.neuzip_decompress(blob, out)
    nz.neuzip_check(blob)
    assert np.array_equal(inputs.bits(out), want_words), f"{what}: decoded"
    return want_container


@pytest.mark.parametrize("n", [1, 9, 4095, 4096, 4097, 16 * 4096 + 13, 33 * 4096 + 2049, 1_000_003])
def test_update_matches_the_oracle_over_several_steps(nz, n):
    w = inputs.gaussian_bf16(n, 10_000 + n % 991, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w], 7, 8)
    container = O.compress(inputs.bits(w), 7, threads=8, guard=8)
    for step, lr in enumerate((1e-3, 3e-4, 1e-3)):
        g = inputs.gaussian_bf16(n, 10_100 + 7 * step + n % 13, std=0.05, device=DEV)
        container = one_step(nz, blob, container, g, lr, f"n={n} step {step}", ready=step)
    g = inputs.gaussian_bf16(n, 10_190 + n % 13, std=0.05, device=DEV)
    one_step(nz, blob, container, g, 1e-3, f"n={n} scratch only", ready=3)


@pytest.mark.parametrize("lr", [0.0, 1e-2, -3.0, 1e-30, 3e38, float("inf")])
def test_update_on_every_weight_pattern(nz, lr):
    # every bf16 pattern as the weight (subnormals, infinities, NaNs), random bit patterns as the gradient
    w = inputs.all_patterns_bf16(device=DEV)
    blob = nz.neuzip_compress(w, 7)
    container = O.compress(inputs.bits(w), 7)
    g = inputs.random_bits_bf16(65536, 10_200, device=DEV)
    one_step(nz, blob, container, g, lr, f"lr={lr}", ready=1)
    # and every pattern as the gradient of ordinary weights
    w2 = inputs.gaussian_bf16(65536, 10_201, device=DEV)
    (blob2,) = nz.neuzip_compress_guarded([w2], 7, 4)
    one_step(nz, blob2, O.compress(inputs.bits(w2), 7, guard=4), inputs.all_patterns_bf16(device=DEV), lr, f"grad lr={lr}",
             ready=2)


@pytest.mark.parametrize("ready", [0, 1, 2, 3])
def test_update_a_layer_in_one_call(nz, ready):
    shapes = [(512, 512), (128, 512), (128, 512), (512, 512), (512, 1792), (512, 1792), (1792, 512), (77, 13), (0,),
              (3, 4096)]
    ws = [inputs.gaussian_bf16(s, 10_300 + i, device=DEV) for i, s in enumerate(shapes)]
    gs = [inputs.gaussian_bf16(s, 10_400 + i, std=0.05, device=DEV) for i, s in enumerate(shapes)]
    # the gradient of tensor 4 holds a value that throws its weight far outside the table
    g4 = inputs.bits(gs[4]).copy()
    g4[4321] = 0xC900                                             # -2^19
    gs[4] = inputs.from_bits(g4, DEV).reshape(shapes[4])
    blobs = nz.neuzip_compress_guarded(ws, 7, 8)
    containers = [O.compress(inputs.bits(w), 7, guard=8) for w in ws]
    spaces = [w.clone() if ready in (1, 2) else torch.full_like(w, float("nan")) for w in ws]
    rebuilt = nz.neuzip_update(blobs, gs, spaces, 1e-3, weights_ready=ready)
    assert rebuilt[4] == 1 and sum(rebuilt) < len(rebuilt)
    for i, (b, c, g, s) in enumerate(zip(blobs, containers, gs, spaces)):
        want_container, want_rebuilt, want_words = U.training_step(c, inputs.bits(g), 1e-3)
        if ready >= 2 and not rebuilt[i]:
            assert np.array_equal(inputs.bits(s), inputs.bits(ws[i])), i
        else:
            assert np.array_equal(inputs.bits(s), want_words), i
        assert want_rebuilt == rebuilt[i], (i, rebuilt)
        same_container(nz.neuzip_export(b), want_container, f"tensor {i}")


def test_update_single_exponent_and_spread_exponents(nz):
    # one exponent value: the decoder's path without words; the step then spreads the exponents
    c = inputs.constant_bf16(50_000, 0.75, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([c], 7, 2)
    g = inputs.gaussian_bf16(50_000, 10_500, std=1.0, device=DEV)
    one_step(nz, blob, O.compress(inputs.bits(c), 7, guard=2), g, 0.5, "single exponent")
    # uniformly random words: over 5 bits per exponent, the decoder reads the words from the blob
    r = inputs.random_bits_bf16(300_000, 10_501, device=DEV)
    blob = nz.neuzip_compress(r, 7)
    one_step(nz, blob, O.compress(inputs.bits(r), 7), inputs.gaussian_bf16(300_000, 10_502, device=DEV), 1e-3, "spread")


def test_update_of_a_tensor_that_streams_to_hbm(nz):
    n = (64 << 20) + 4096 + 77
    w = inputs.gaussian_bf16(n, 10_600, device=DEV)
    g = inputs.gaussian_bf16(n, 10_601, std=0.05, device=DEV)
    (blob,) = nz.neuzip_compress_guarded([w], 7, 8)
    space = torch.empty_like(w)
    (rebuilt,) = nz.neuzip_update([blob], [g], [space], 1e-3)
    want = U.sgd_update(inputs.bits(w), inputs.bits(g), 1e-3)
    assert np.array_equal(inputs.bits(space), want)
    table = nz.neuzip_frequencies(blob)
    assert rebuilt == 0
    same_container(nz.neuzip_export(blob), O.compress(want, 7, threads=8, guard=8, freq=table), "streaming size")


def test_update_argument_errors(nz):
    w = inputs.gaussian_bf16(10_000, 10_700, device=DEV)
    g = inputs.gaussian_bf16(10_000, 10_701, device=DEV)
    s = torch.empty_like(w)
    (blob,) = nz.neuzip_compress_guarded([w], 7, 8)
    before = nz.neuzip_export(blob)
    lossy = nz.neuzip_compress(w, 3)
    with pytest.raises(nz.NeuzipError) as err:
        nz.neuzip_update([lossy], [g], [s], 1e-3)
    assert err.value.code == nz.EUNSUPPORTED
    wide = nz.neuzip_compress(w.float(), 7)
    lib = nz.library()
    one = lambda h: (ctypes.c_void_p * 1)(h)
    call = lambda handle, gp, wp: lib.neuzip_update(one(handle), one(gp), one(wp), 1, 1e-3, 0, None, None)
    assert call(wide.handle.value, g.data_ptr(), s.data_ptr()) == nz.EUNSUPPORTED
    assert call(blob.handle.value, g.data_ptr() + 2, s.data_ptr()) == nz.EINVAL      # misaligned gradient
    assert call(blob.handle.value, g.data_ptr(), None) == nz.EINVAL
    assert call(blob.handle.value, g.data_ptr(), g.data_ptr()) == nz.EINVAL          # the step cannot run over its own gradient
    assert call(None, g.data_ptr(), s.data_ptr()) == nz.EINVAL
    two = (ctypes.c_void_p * 2)(blob.handle.value, blob.handle.value)
    gp = (ctypes.c_void_p * 2)(g.data_ptr(), g.data_ptr())
    wp = (ctypes.c_void_p * 2)(s.data_ptr(), s.data_ptr())
    assert lib.neuzip_update(two, gp, wp, 2, 1e-3, 0, None, None) == nz.EINVAL          # one blob twice
    assert lib.neuzip_update(one(blob.handle.value), one(g.data_ptr()), one(s.data_ptr()), 1, 1e-3, 4, None, None) == nz.EINVAL
    with pytest.raises(ValueError):
        nz.neuzip_update([blob], [g[:100].contiguous()], [s], 1e-3)
    assert np.array_equal(nz.neuzip_export(blob), before)                            # untouched by the failed calls
