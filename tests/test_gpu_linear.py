"""GPU parity of the fused decode + matrix-core linear layer (-m gpu).

Sec. 2.2, compressed forward pass: W_hat <- decompress(c_l); x_l <- W_hat x_{l-1} + b_l.  The
oracle evaluates that definition in float64 (oracle/linear.py).  The kernel multiplies bf16 values
exactly and sums in float32, in an order of its own (matrix-core accumulation over 32 input
features at a time, then float atomics across the pieces of a row), so the bar is the classical
bound for a float32 sum of N terms in any order: |error| <= N * 2^-24 * sum |w_k x_k|, with N =
in_features + the number of partial sums; the tests allow twice that.
"""
import numpy as np
import pytest
import torch

from oracle import linear as L
from oracle import oracle as O
from paper_2410_20650_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def nz():
    from paper_2410_20650_amd import binding
    return binding


def check_linear(nz, w, out_f, in_f, tokens, k=7, bias=False, seed=1, block=0):
    """Compress w (flat bf16, out_f * in_f) on the GPU, run the fused layer, compare with the oracle."""
    x = inputs.gaussian_bf16((tokens, in_f), seed, std=1.0, device=DEV)
    b = (torch.arange(out_f, dtype=torch.float32, device=DEV) * 0.37 - 2.0) if bias else None
    blob = nz.neuzip_compress_blockwise(w, k, block)
    y = torch.full((tokens, out_f), float("nan"), dtype=torch.float32, device=DEV)
    nz.neuzip_linear(blob, out_f, in_f, x, b, y)
    nz.neuzip_check(blob)
    container = O.compress(inputs.bits(w), k, threads=8, block=block)   # the oracle's own container of the same weight
    xw = inputs.bits(x).reshape(tokens, in_f)
    want = L.linear(container, out_f, in_f, xw, bias=None if b is None else b.cpu().numpy().astype(np.float64))
    mag = L.magnitude(container, out_f, in_f, xw)
    if b is not None:
        mag = mag + np.abs(b.cpu().numpy().astype(np.float64))
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    bound = 2.0 * (in_f + 64) * 2.0 ** -24 * mag + 1e-30
    worst = np.max(np.abs(got - want) / bound)
    assert worst <= 1.0, f"error {worst:.3f} x the float32 bound (out={out_f}, in={in_f}, tokens={tokens}, k={k})"
    return blob, x, y


@pytest.mark.parametrize("tokens", [1, 5, 16, 17, 33, 64])
@pytest.mark.parametrize("out_f,in_f", [(16, 128), (40, 256), (64, 4096), (37, 4096), (48, 14336), (33, 11008),
                                        (8, 8192)])
def test_linear_matches_the_oracle(nz, out_f, in_f, tokens):
    w = inputs.gaussian_bf16(out_f * in_f, 9000 + out_f + in_f, device=DEV)
    check_linear(nz, w, out_f, in_f, tokens, seed=9100 + tokens)


@pytest.mark.parametrize("k", [3, 1, 0])
def test_linear_on_lossy_weights_uses_the_truncated_values(nz, k):
    out_f, in_f = 96, 1024
    w = inputs.student_t4_bf16(out_f * in_f, 9200 + k, device=DEV)
    check_linear(nz, w, out_f, in_f, 9, k=k, bias=True, seed=9201)


@pytest.mark.parametrize("k,block", [(3, 512), (3, 32), (1, 64), (0, 512), (0, 128)])
def test_linear_on_blockwise_normalised_weights(nz, k, block):
    # the paper's default lossy form (block-wise normalisation): the layer multiplies bf16(stored * c)
    for out_f, in_f, tokens in ((96, 1024, 9), (37, 4096, 17), (16, 14336, 33)):
        w = inputs.student_t4_bf16(out_f * in_f, 9400 + k + block, device=DEV)
        check_linear(nz, w, out_f, in_f, tokens, k=k, bias=True, seed=9401, block=block)


@pytest.mark.parametrize("tokens", [65, 128, 200])
def test_linear_on_more_than_64_tokens_goes_through_in_tiles(nz, tokens):
    for out_f, in_f, k, block in ((40, 256, 7, 0), (64, 4096, 7, 0), (48, 14336, 3, 0), (33, 1024, 0, 512)):
        w = inputs.gaussian_bf16(out_f * in_f, 9500 + out_f, device=DEV)
        check_linear(nz, w, out_f, in_f, tokens, k=k, bias=True, seed=9501 + tokens, block=block)


@pytest.mark.parametrize("tokens", [1, 8, 40, 100])
@pytest.mark.parametrize("k,block", [(7, 0), (3, 0), (0, 512)])
def test_linear_batch_of_projections_matches_the_oracle_and_the_single_calls(nz, tokens, k, block):
    # the q, k and v projections of an attention block on the same activations, in one launch
    in_f, outs = 1024, (256, 64, 37)
    ws = [inputs.gaussian_bf16(o * in_f, 9800 + o, device=DEV) for o in outs]
    x = inputs.gaussian_bf16((tokens, in_f), 9801 + tokens, std=1.0, device=DEV)
    biases = [torch.linspace(-1, 1, outs[0], dtype=torch.float32, device=DEV), None,
              torch.linspace(2, 3, outs[2], dtype=torch.float32, device=DEV)]
    blobs = [nz.neuzip_compress_blockwise(w, k, block) for w in ws]
    ys = [torch.full((tokens, o), float("nan"), dtype=torch.float32, device=DEV) for o in outs]
    nz.neuzip_linear_batch(blobs, outs, in_f, x, biases, ys)
    xw = inputs.bits(x).reshape(tokens, in_f)
    for w, blob, o, bias, y in zip(ws, blobs, outs, biases, ys):
        nz.neuzip_check(blob)
        container = O.compress(inputs.bits(w), k, threads=8, block=block)
        b64 = None if bias is None else bias.cpu().numpy().astype(np.float64)
        want = L.linear(container, o, in_f, xw, bias=b64)
        mag = L.magnitude(container, o, in_f, xw) + (0 if b64 is None else np.abs(b64))
        got = y.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got))
        bound = 2.0 * (in_f + 64) * 2.0 ** -24 * mag + 1e-30
        assert np.max(np.abs(got - want) / bound) <= 1.0, (o, tokens, k, block)
        single = nz.neuzip_linear(blob, o, in_f, x, bias)
        assert torch.allclose(y, single, rtol=0, atol=1e-5 * max(single.abs().max().item(), 1e-30))


def test_linear_batch_argument_errors(nz):
    in_f = 256
    w7 = nz.neuzip_compress(inputs.gaussian_bf16(32 * in_f, 9810, device=DEV), 7)
    w3 = nz.neuzip_compress(inputs.gaussian_bf16(32 * in_f, 9811, device=DEV), 3)
    x = inputs.gaussian_bf16((4, in_f), 9812, device=DEV)
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_linear_batch([w7, w3], [32, 32], in_f, x)            # mixed mantissa widths
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_linear_batch([w7] * 5, [32] * 5, in_f, x)            # more than 4 weights
    with pytest.raises(nz.NeuzipError):
        nz.neuzip_linear_batch([w7, w7], [32, 16], in_f, x)            # shape does not match the blob
    assert nz.neuzip_linear_batch([], [], in_f, x) == []
    ys = nz.neuzip_linear_batch([w7, w7], [32, 32], in_f, x)
    assert torch.equal(ys[0], ys[1]) or torch.allclose(ys[0], ys[1], rtol=0, atol=1e-6)
    torch.cuda.synchronize()


def test_linear_with_bias_and_one_hot_activations(nz):
    # one-hot activations select weight columns: the result is exact, whatever the summation order
    out_f, in_f = 50, 512
    w = inputs.gaussian_bf16(out_f * in_f, 9300, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    picks = [0, 7, 8, 127, 128, 300, 511]
    x = torch.zeros((len(picks), in_f), dtype=torch.bfloat16, device=DEV)
    for t, kcol in enumerate(picks):
        x[t, kcol] = 1.0
    bias = torch.linspace(-1, 1, out_f, dtype=torch.float32, device=DEV)
    y = nz.neuzip_linear(blob, out_f, in_f, x, bias)
    wf = w.float().reshape(out_f, in_f)
    for t, kcol in enumerate(picks):
        assert torch.equal(y[t], wf[:, kcol] + bias)


def test_linear_single_exponent_and_wide_exponent_weights(nz):
    # one exponent value: the decoder's path without words
    out_f, in_f = 24, 512
    sign = torch.where(torch.arange(out_f * in_f, device=DEV) % 3 == 0, -1.0, 1.0)
    w = (sign * 0.75).to(torch.bfloat16)
    check_linear(nz, w, out_f, in_f, 4, seed=9400)
    # exponents spread over 40 values (over 5 bits per symbol): the word runs do not fit the LDS
    # window and are read from the blob
    g = torch.Generator(device=DEV).manual_seed(9401)
    n = 64 * 2048
    expo = torch.randint(100, 140, (n,), generator=g, device=DEV, dtype=torch.int32)
    rest = torch.randint(0, 256, (n,), generator=g, device=DEV, dtype=torch.int32)
    words = ((rest & 0x80) << 8) | (expo << 7) | (rest & 0x7F)
    w = (words - 65536 * (words >= 32768)).to(torch.int16).view(torch.bfloat16)
    check_linear(nz, w, 64, 2048, 20, seed=9402)


def test_linear_full_projection_shape(nz):
    # a q/o projection of Llama-3 8B at full size, a decoding batch of 8 tokens
    out_f = in_f = 4096
    w = inputs.gaussian_bf16(out_f * in_f, inputs.seed_for(3, 1), device=DEV)
    blob, x, y = check_linear(nz, w, out_f, in_f, 8, seed=9500)
    # against the dense product of the decompressed weight on the GPU (bf16 inputs, float32 sums)
    dense = torch.empty(out_f * in_f, dtype=torch.bfloat16, device=DEV)
    nz.neuzip_decompress(blob, dense)
    ref = x.float() @ dense.float().reshape(out_f, in_f).T
    assert torch.allclose(y, ref, rtol=0, atol=2e-3 * ref.abs().max().item())


def test_linear_on_the_largest_weight_of_the_model(nz):
    # the output projection of Llama-3 8B (128256 x 4096, 525 M elements) applied to a decoding batch.
    # Every output against the dense float32 product of the decompressed weight on the GPU; a sample of
    # rows against the definition (Sec. 2.2: W_hat x with W_hat = decompress(c), which for a lossless
    # blob is the weight itself) in float64, within the float32 summation bound.
    out_f, in_f, tokens = 128256, 4096, 8
    w = inputs.gaussian_bf16((out_f, in_f), inputs.seed_for(3, 0), device=DEV)
    x = inputs.gaussian_bf16((tokens, in_f), 9900, std=1.0, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    y = nz.neuzip_linear(blob, out_f, in_f, x)
    nz.neuzip_check(blob)
    dense = torch.empty_like(w)
    nz.neuzip_decompress(blob, dense.view(-1))
    assert torch.equal(dense.view(torch.int16), w.view(torch.int16))
    ref = x.float() @ dense.float().T
    assert torch.allclose(y, ref, rtol=0, atol=2e-3 * ref.abs().max().item())
    rows = torch.linspace(0, out_f - 1, 257, device=DEV).long()
    w64 = w[rows].double().cpu().numpy()
    x64 = x.double().cpu().numpy()
    want = x64 @ w64.T
    mag = np.abs(x64) @ np.abs(w64).T
    got = y[:, rows].cpu().numpy().astype(np.float64)
    bound = 2.0 * (in_f + 64) * 2.0 ** -24 * mag + 1e-30
    assert np.max(np.abs(got - want) / bound) <= 1.0
    nz.neuzip_free(blob)


def test_linear_argument_errors(nz):
    w = inputs.gaussian_bf16(32 * 256, 9600, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    x = inputs.gaussian_bf16((4, 256), 9601, device=DEV)
    lib = nz.library()
    import ctypes
    y = torch.zeros((4, 64), dtype=torch.float32, device=DEV)
    args = lambda out_f, in_f, tokens: (blob.handle, out_f, in_f, ctypes.c_void_p(x.data_ptr()), tokens, None,
                                        ctypes.c_void_p(y.data_ptr()), None)
    assert lib.neuzip_linear(*args(32, 256, 4)) == nz.OK
    assert lib.neuzip_linear(*args(16, 256, 4)) == nz.EINVAL       # shape does not match the blob
    assert lib.neuzip_linear(*args(64, 128, 4)) == nz.OK           # same elements, another valid shape
    assert lib.neuzip_linear(*args(128, 64, 4)) == nz.EINVAL       # in_features not a multiple of 128
    assert lib.neuzip_linear(*args(32, 256, 0)) == nz.EINVAL
    assert lib.neuzip_linear(None, 32, 256, ctypes.c_void_p(x.data_ptr()), 4, None, ctypes.c_void_p(y.data_ptr()),
                             None) == nz.EINVAL
    w32 = nz.neuzip_compress(inputs.gaussian_f32(32 * 256, 9602, device=DEV), 7)
    assert lib.neuzip_linear(w32.handle, 32, 256, ctypes.c_void_p(x.data_ptr()), 4, None,
                             ctypes.c_void_p(y.data_ptr()), None) == nz.EUNSUPPORTED   # bf16 weights only
    torch.cuda.synchronize()


def test_linear_can_be_captured_in_a_hip_graph(nz):
    # the fused layer allocates nothing and clears y with a kernel, not a memset node: a decoding
    # step can be captured once and replayed; every replay is checked against the eager result
    out_f, in_f, tokens = 256, 4096, 4
    w = inputs.gaussian_bf16(out_f * in_f, 9700, device=DEV)
    blob = nz.neuzip_compress(w, 7)
    x = inputs.gaussian_bf16((tokens, in_f), 9701, std=1.0, device=DEV)
    bias = torch.linspace(-1, 1, out_f, dtype=torch.float32, device=DEV)
    y = torch.zeros((tokens, out_f), dtype=torch.float32, device=DEV)
    eager = nz.neuzip_linear(blob, out_f, in_f, x, bias).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        nz.neuzip_linear(blob, out_f, in_f, x, bias, y, stream=side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            nz.neuzip_linear(blob, out_f, in_f, x, bias, y, stream=side)
    for replay in range(4):
        y.fill_(float("nan"))                                       # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        # the order of the float atomics may differ from run to run: a few ulps of the sums
        assert torch.allclose(y, eager, rtol=0, atol=1e-5 * eager.abs().max().item()), replay
    nz.neuzip_check(blob)
