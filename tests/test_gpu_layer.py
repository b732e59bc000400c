"""The layer-by-layer training step of Alg. 1 on compressed weights (-m gpu).

The dense products are torch's and are checked within their rounding (bf16 results of float32
accumulations); everything the codec does is checked exactly: after each layer's update the blob
must be the container that oracle/update.py derives from the container before, the gradient that
was applied and the rate.
"""
import numpy as np
import pytest
import torch

from oracle import linear as L
from oracle import oracle as O
from oracle import update as U
from paper_2410_20650_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def nz():
    from paper_2410_20650_amd import binding
    return binding


def as_f64(t):
    return L.bf16_to_float64(inputs.bits(t)).reshape(tuple(t.shape))


@pytest.mark.parametrize("tokens", [8, 200])
def test_training_steps_follow_alg1(nz, tokens):
    from paper_2410_20650_amd import layer
    dims = [256, 512, 384, 128]
    ws = [inputs.gaussian_bf16((dims[i + 1], dims[i]), 11_000 + i, std=0.05, device=DEV) for i in range(3)]
    layers = [layer.CompressedLinear(w, guard=8) for w in ws]
    containers = [O.compress(inputs.bits(w), 7, guard=8) for w in ws]
    space = torch.empty(512 * 384, dtype=torch.bfloat16, device=DEV)
    grad_space = torch.empty_like(space)
    x = inputs.gaussian_bf16((tokens, dims[0]), 11_010, std=1.0, device=DEV)
    target = inputs.gaussian_bf16((tokens, dims[-1]), 11_011, std=1.0, device=DEV)
    lr = 1e-3 / tokens
    losses = []
    for step in range(3):
        # forward pass of every layer against the float64 definition, from the containers as they stand
        h = x
        for i, c in enumerate(containers):
            w = L.bf16_to_float64(O.decompress(c, dims[i + 1] * dims[i])).reshape(dims[i + 1], dims[i])
            want = as_f64(h) @ w.T
            scale = np.abs(as_f64(h)) @ np.abs(w).T
            got = layers[i].forward(h, space)
            # the fused kernel returns float32 sums; the dense route (more than 64 tokens) a bf16 product
            rounding = 0.0 if tokens <= 64 else 2.0 ** -8
            assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want)
                          <= rounding * np.abs(want) + (dims[i] + 64) * 2.0 ** -23 * scale + 1e-30), (step, i)
            h = (torch.relu(got) if i < 2 else got).to(torch.bfloat16)

        seen = {}

        def observer(i, layer_input, grad_y, grad_w):
            # the weight gradient against its definition, within the bf16 rounding of a float32 sum
            want = as_f64(grad_y).T @ as_f64(layer_input)
            mag = np.abs(as_f64(grad_y)).T @ np.abs(as_f64(layer_input))
            assert np.all(np.abs(as_f64(grad_w) - want) <= 2.0 ** -8 * np.abs(want) + 2.0 ** -18 * mag + 1e-30), i
            now = torch.empty(grad_w.numel(), dtype=torch.bfloat16, device=DEV)
            nz.neuzip_decompress(layers[i].blob, now)
            seen[i] = (inputs.bits(grad_w).copy(), nz.neuzip_export(layers[i].blob), inputs.bits(now))

        loss, flags = layer.training_step(layers, x, target, lr, space, grad_space, observer=observer)
        losses.append(loss)
        # the exact part: each blob is the oracle's container for the gradient that was applied
        for i in range(3):
            grad_bits, got, new_words = seen[i]
            want_container, rebuilt, want_words = U.training_step(containers[i], grad_bits, lr, threads=8)
            assert rebuilt == flags[i]
            assert np.array_equal(new_words, want_words), (step, i)
            assert got.size == want_container.size and np.array_equal(got, want_container), (step, i)
            containers[i] = want_container
    assert losses[2] < losses[0]                                         # the steps reduce the loss
