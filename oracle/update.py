"""The weight update of the compressed training loop, as the plain definition (test infrastructure only).

Alg. 1, backward loop: for each layer the weight is decompressed into temporary space, its
gradient is computed, the optimiser step is applied and the weight is compressed again:
    W_hat <- decompress(c_l);   W_hat <- W_hat - lr * grad_W;   c_l <- compress(W_hat)
(Sec. 2.2 uses the update rule of vanilla SGD applied layer by layer during the backward pass.)
The paper does not state the precision of the step.  Reading taken here: every element is
updated in IEEE binary32 -- the product lr * g rounded to binary32, then the difference rounded
to binary32, no fused multiply-add -- and the result is rounded to the nearest bf16, ties to even.
A NaN result is stored as the quiet NaN 0x7FC0.  numpy's float32 arithmetic performs exactly
these roundings; the last rounding is written out on the integer representation.

Only tests, the smoke check and the benchmark's CPU-baseline leg may call this.  It shares no
code with the HIP library.
"""
import numpy as np

from . import oracle as O


def round_to_bf16(values):
    """binary32 values -> bf16 words, round to nearest, ties to even; NaN -> 0x7FC0."""
    v = np.ascontiguousarray(values, dtype=np.float32)
    b = v.view(np.uint32).astype(np.uint64)
    # add half an ulp of the upper half, less one when the kept part is even: the carry rounds
    rounded = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
    return np.where(np.isnan(v), np.uint16(0x7FC0), rounded)


def sgd_update(w_words, g_words, lr):
    """bf16 words of W - lr * G for bf16 words of W and G (element by element)."""
    w = (np.ascontiguousarray(w_words, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
    g = (np.ascontiguousarray(g_words, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
    with np.errstate(all="ignore"):
        step = np.float32(lr) * g          # rounded to binary32
        new = w - step                      # rounded to binary32
    return round_to_bf16(new)


def training_step(container, g_words, lr, threads=1):
    """One pass of the backward loop for one weight: (new container, rebuilt flag, new bf16 words).

    The new tensor is coded with the table the container holds; if that table has no room for an
    exponent the update produced, the tensor is compressed with fresh statistics and the
    container's guard band, and the flag is 1."""
    info = O.blob_info(container)
    if info["k"] != 7:
        raise ValueError("training works on lossless containers")
    new = sgd_update(O.decompress(container, info["n"], threads=threads), g_words, lr)
    guard = int(np.ascontiguousarray(container[52:56]).view("<u4")[0])
    try:
        return O.compress(new, 7, threads=threads, guard=guard, freq=info["freq"]), 0, new
    except O.OracleError as err:
        if err.code != O.ESTALE:
            raise
    return O.compress(new, 7, threads=threads, guard=guard), 1, new
