"""The linear layer on a compressed weight, as the plain definition (test infrastructure only).

Sec. 2.2, the compressed forward pass: W_hat <- decompress(c_l);  x_l <- W_hat x_{l-1} + b_l.
The weight matrix is out_features x in_features, stored row by row as the flat bf16 tensor that
was compressed; the activations are bf16, one row per token.  Everything is evaluated in
float64 (every bf16 value and every product of two is exact there; only the sum over
in_features rounds, at 2^-53 relative to the magnitudes summed).  A library matrix product is
the one step used; there is no blocking or reordering.

Only tests, the smoke check and the benchmark's CPU-baseline leg may call this.  It shares no
code with the HIP library.
"""
import numpy as np

from . import oracle as O


def bf16_to_float64(words):
    """The real numbers that bf16 words denote (bf16 is the upper half of IEEE binary32)."""
    words = np.ascontiguousarray(words, dtype=np.uint16)
    with np.errstate(invalid="ignore"):
        return (words.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def linear(container, out_features, in_features, x_words, bias=None, threads=1):
    """y[t][o] = sum_k W_hat[o][k] * x[t][k] + b[o], float64, shape (tokens, out_features).

    container: the compressed weight (bytes as a uint8 array); x_words: bf16 words of the
    activations, shape (tokens, in_features); bias: float values per output feature or None."""
    n = out_features * in_features
    w_hat = bf16_to_float64(O.decompress(container, n, threads=threads)).reshape(out_features, in_features)
    x = bf16_to_float64(x_words).reshape(-1, in_features)
    y = x @ w_hat.T
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, out_features)
    return y


def magnitude(container, out_features, in_features, x_words, threads=1):
    """sum_k |W_hat[o][k]| * |x[t][k]|: the scale against which a float32 accumulation is judged."""
    n = out_features * in_features
    w_hat = np.abs(bf16_to_float64(O.decompress(container, n, threads=threads))).reshape(out_features, in_features)
    x = np.abs(bf16_to_float64(x_words)).reshape(-1, in_features)
    return x @ w_hat.T
