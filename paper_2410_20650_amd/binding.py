"""Thin ctypes binding of libneuzip.so: argument marshalling only.

Every step of the method runs inside the HIP library; PyTorch is used for
device memory and streams.  The functions mirror include/neuzip.h name for
name.  If the library has not been built it is built once with hipcc; if that
is impossible the import fails loudly -- there is no CPU fallback.
"""
import ctypes
import os

import numpy as np
import torch

from . import build as _build

BF16, F32, F16 = 0, 1, 2
OK, EINVAL, ENOMEM, EHIP, ECORRUPT, EUNSUPPORTED = 0, -1, -2, -3, -4, -5


class NeuzipError(RuntimeError):
    def __init__(self, code, what):
        msg = _lib.neuzip_strerror(code).decode() if _lib is not None else "?"
        hip = _lib.neuzip_last_hip_error() if _lib is not None else 0
        super().__init__(f"{what}: {msg} (code {code}, hip error {hip})")
        self.code = code


def _load():
    if not os.path.exists(_build.LIB):
        _build.build()
    lib = ctypes.CDLL(_build.LIB)
    vp, u64, i32, u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_uint32
    vpp = ctypes.POINTER(vp)
    lib.neuzip_compress.argtypes = [vp, u64, i32, i32, vp, vpp]
    lib.neuzip_compress.restype = i32
    lib.neuzip_compress_noalloc.argtypes = [vp, u64, i32, i32, vp, vp]
    lib.neuzip_compress_noalloc.restype = i32
    lib.neuzip_compress_blockwise.argtypes = [vp, u64, i32, i32, u32, vp, vpp]
    lib.neuzip_compress_blockwise.restype = i32
    lib.neuzip_compress_batch.argtypes = [vpp, ctypes.POINTER(u64), u32, i32, i32, u32, vp, vpp]
    lib.neuzip_compress_batch.restype = i32
    lib.neuzip_compress_guarded.argtypes = [vpp, ctypes.POINTER(u64), u32, i32, i32, u32, vp, vpp]
    lib.neuzip_compress_guarded.restype = i32
    lib.neuzip_recompress.argtypes = [vpp, u32, vp, vpp, ctypes.POINTER(u32)]
    lib.neuzip_recompress.restype = i32
    lib.neuzip_update.argtypes = [vpp, vpp, vpp, u32, ctypes.c_float, i32, vp, ctypes.POINTER(u32)]
    lib.neuzip_update.restype = i32
    lib.neuzip_linear.argtypes = [vp, u64, u64, vp, u32, vp, vp, vp]
    lib.neuzip_linear.restype = i32
    lib.neuzip_linear_batch.argtypes = [vp, vp, u32, u64, vp, u32, vp, vp, vp]
    lib.neuzip_linear_batch.restype = i32
    lib.neuzip_block_size.argtypes = [vp]
    lib.neuzip_block_size.restype = u32
    lib.neuzip_guard.argtypes = [vp]
    lib.neuzip_guard.restype = u32
    lib.neuzip_decompress.argtypes = [vp, vp, u64, i32, vp]
    lib.neuzip_decompress.restype = i32
    lib.neuzip_decompress_sequence.argtypes = [vpp, u32, vp, u64, ctypes.POINTER(u64), vp]
    lib.neuzip_decompress_sequence.restype = i32
    lib.neuzip_decompress_batch.argtypes = [vpp, vpp, u32, vp]
    lib.neuzip_decompress_batch.restype = i32
    lib.neuzip_free.argtypes = [vp]
    lib.neuzip_free.restype = None
    lib.neuzip_compressed_bytes.argtypes = [vp]
    lib.neuzip_compressed_bytes.restype = u64
    lib.neuzip_device_bytes.argtypes = [vp]
    lib.neuzip_device_bytes.restype = u64
    lib.neuzip_elems.argtypes = [vp]
    lib.neuzip_elems.restype = u64
    lib.neuzip_mantissa_bits.argtypes = [vp]
    lib.neuzip_mantissa_bits.restype = i32
    lib.neuzip_dtype.argtypes = [vp]
    lib.neuzip_dtype.restype = i32
    lib.neuzip_export.argtypes = [vp, vp, u64, ctypes.POINTER(u64), vp]
    lib.neuzip_export.restype = i32
    lib.neuzip_import.argtypes = [vp, u64, vp, vpp]
    lib.neuzip_import.restype = i32
    lib.neuzip_histogram.argtypes = [vp, ctypes.POINTER(u32)]
    lib.neuzip_histogram.restype = i32
    lib.neuzip_frequencies.argtypes = [vp, ctypes.POINTER(ctypes.c_uint16)]
    lib.neuzip_frequencies.restype = i32
    lib.neuzip_stream_probe.argtypes = [vp, u64, vp, u64, vp]
    lib.neuzip_stream_probe.restype = i32
    lib.neuzip_check.argtypes = [vp, vp]
    lib.neuzip_check.restype = i32
    lib.neuzip_workspace_bytes.argtypes = []
    lib.neuzip_workspace_bytes.restype = u64
    lib.neuzip_release_workspace.argtypes = []
    lib.neuzip_release_workspace.restype = i32
    lib.neuzip_set_workspace_limit.argtypes = [u64]
    lib.neuzip_set_workspace_limit.restype = i32
    lib.neuzip_strerror.argtypes = [i32]
    lib.neuzip_strerror.restype = ctypes.c_char_p
    lib.neuzip_last_hip_error.argtypes = []
    lib.neuzip_last_hip_error.restype = i32
    return lib


_lib = None
_lib = _load()

EXPORTED = ["neuzip_compress", "neuzip_compress_noalloc", "neuzip_compress_blockwise", "neuzip_compress_batch", "neuzip_compress_guarded",
            "neuzip_recompress", "neuzip_update", "neuzip_guard", "neuzip_linear", "neuzip_linear_batch", "neuzip_block_size", "neuzip_decompress", "neuzip_decompress_sequence", "neuzip_decompress_batch",
            "neuzip_free",
            "neuzip_compressed_bytes", "neuzip_device_bytes", "neuzip_elems", "neuzip_mantissa_bits", "neuzip_dtype",
            "neuzip_export", "neuzip_import", "neuzip_histogram", "neuzip_frequencies", "neuzip_check", "neuzip_stream_probe",
            "neuzip_workspace_bytes", "neuzip_release_workspace", "neuzip_set_workspace_limit", "neuzip_strerror", "neuzip_last_hip_error"]


def library():
    return _lib


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_tensor(t, wide_ok=False):
    """Returns the library's element type of a contiguous CUDA tensor (bf16; float32 and float16 where allowed)."""
    if t.is_cuda and t.is_contiguous():
        if t.dtype == torch.bfloat16:
            return BF16
        if wide_ok and t.dtype == torch.float32:
            return F32
        if wide_ok and t.dtype == torch.float16:
            return F16
    raise TypeError("expected a contiguous bf16%s CUDA tensor" % (", float32 or float16" if wide_ok else ""))


def _shared_dtype(tensors):
    kinds = {_check_tensor(t, wide_ok=True) for t in tensors}
    if len(kinds) > 1:
        raise TypeError("the tensors of one call share one element type")
    return kinds.pop() if kinds else BF16


class Blob:
    """Owns one neuzip_blob handle."""

    def __init__(self, handle):
        self.handle = ctypes.c_void_p(handle)

    def free(self):
        if self.handle:
            _lib.neuzip_free(self.handle)
            self.handle = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    @property
    def compressed_bytes(self):
        return int(_lib.neuzip_compressed_bytes(self.handle))

    @property
    def device_bytes(self):
        return int(_lib.neuzip_device_bytes(self.handle))

    @property
    def elems(self):
        return int(_lib.neuzip_elems(self.handle))

    @property
    def mantissa_bits(self):
        return int(_lib.neuzip_mantissa_bits(self.handle))

    @property
    def block_size(self):
        return int(_lib.neuzip_block_size(self.handle))

    @property
    def guard(self):
        return int(_lib.neuzip_guard(self.handle))

    @property
    def dtype(self):
        return int(_lib.neuzip_dtype(self.handle))


def neuzip_compress(src: torch.Tensor, mantissa_bits: int = 7, stream=None, blob: Blob = None) -> Blob:
    return neuzip_compress_blockwise(src, mantissa_bits, 0, stream, blob)


def neuzip_compress_noalloc(src: torch.Tensor, mantissa_bits: int, blob: Blob, stream=None) -> Blob:
    """neuzip_compress into an existing blob through the library's fixed workspace (allocates nothing)."""
    dtype = _check_tensor(src, wide_ok=True)
    rc = _lib.neuzip_compress_noalloc(ctypes.c_void_p(src.data_ptr()), src.numel(), dtype, mantissa_bits,
                                      _stream_handle(stream), blob.handle)
    if rc != OK:
        raise NeuzipError(rc, "neuzip_compress_noalloc")
    return blob


def neuzip_compress_blockwise(src: torch.Tensor, mantissa_bits: int, block_size: int, stream=None,
                              blob: Blob = None) -> Blob:
    dtype = _check_tensor(src, wide_ok=True)
    handle = ctypes.c_void_p(blob.handle.value if blob is not None else None)
    rc = _lib.neuzip_compress_blockwise(ctypes.c_void_p(src.data_ptr()), src.numel(), dtype, mantissa_bits,
                                        block_size, _stream_handle(stream), ctypes.byref(handle))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_compress")
    if blob is not None:
        blob.handle = handle
        return blob
    return Blob(handle.value)


def neuzip_compress_guarded(srcs, mantissa_bits: int = 7, guard: int = 0, stream=None, blobs=None):
    """neuzip_compress_batch with a guard band in the table (for blobs that will be recompressed)."""
    return neuzip_compress_batch(srcs, mantissa_bits, 0, stream, blobs, guard=guard)


def neuzip_recompress(srcs, blobs, stream=None):
    """Codes srcs[i] into blobs[i] with the table the blob holds; returns the list of rebuilt flags."""
    if len(blobs) != len(srcs) or any(b.elems != t.numel() or b.dtype != _check_tensor(t, wide_ok=True)
                                      for b, t in zip(blobs, srcs)):
        raise ValueError("one blob of matching size and element type per tensor")
    count = len(srcs)
    ptrs = (ctypes.c_void_p * count)(*[t.data_ptr() for t in srcs])
    handles = (ctypes.c_void_p * count)(*[b.handle.value for b in blobs])
    rebuilt = (ctypes.c_uint32 * count)()
    rc = _lib.neuzip_recompress(ptrs, count, _stream_handle(stream), handles, rebuilt)
    if rc != OK:
        raise NeuzipError(rc, "neuzip_recompress")
    return [int(v) for v in rebuilt]


def neuzip_update(blobs, grads, weights, lr: float, weights_ready=False, stream=None):
    """blobs[i] <- compress(decompress(blobs[i]) - lr * grads[i]); weights[i] receives the new weight.
    weights_ready: False / 0 -- the library decompresses; True / 1 -- weights[i] already holds
    decompress(blobs[i]); 2 -- the same, and the new weights are not written back; 3 -- the library
    decompresses and weights[i] is mere scratch space.  Returns the list of rebuilt flags."""
    for t in list(grads) + list(weights):
        _check_tensor(t)
    if not (len(blobs) == len(grads) == len(weights)) or any(
            b.elems != g.numel() or b.elems != w.numel() for b, g, w in zip(blobs, grads, weights)):
        raise ValueError("one gradient and one temporary tensor of matching size per blob")
    count = len(blobs)
    handles = (ctypes.c_void_p * count)(*[b.handle.value for b in blobs])
    gptrs = (ctypes.c_void_p * count)(*[g.data_ptr() for g in grads])
    wptrs = (ctypes.c_void_p * count)(*[w.data_ptr() for w in weights])
    rebuilt = (ctypes.c_uint32 * count)()
    rc = _lib.neuzip_update(handles, gptrs, wptrs, count, lr, int(weights_ready), _stream_handle(stream), rebuilt)
    if rc != OK:
        raise NeuzipError(rc, "neuzip_update")
    return [int(v) for v in rebuilt]


def neuzip_compress_batch(srcs, mantissa_bits: int = 7, block_size: int = 0, stream=None, blobs=None, guard=None):
    """Compresses several tensors with one pass of the pipeline; returns one Blob per tensor."""
    dtype = _shared_dtype(srcs)
    if blobs is not None and len(blobs) != len(srcs):
        raise ValueError("one blob per tensor")
    count = len(srcs)
    ptrs = (ctypes.c_void_p * count)(*[t.data_ptr() for t in srcs])
    sizes = (ctypes.c_uint64 * count)(*[t.numel() for t in srcs])
    handles = (ctypes.c_void_p * count)(*[(b.handle.value if b is not None else None)
                                          for b in (blobs if blobs is not None else [None] * count)])
    if guard is None:
        rc = _lib.neuzip_compress_batch(ptrs, sizes, count, dtype, mantissa_bits, block_size, _stream_handle(stream),
                                        handles)
    else:
        rc = _lib.neuzip_compress_guarded(ptrs, sizes, count, dtype, mantissa_bits, guard, _stream_handle(stream),
                                          handles)
    if rc != OK:
        raise NeuzipError(rc, "neuzip_compress_batch")
    out = []
    for i in range(count):
        if blobs is not None and blobs[i] is not None:
            blobs[i].handle = ctypes.c_void_p(handles[i])
            out.append(blobs[i])
        else:
            out.append(Blob(handles[i]))
    return out


def neuzip_decompress(blob: Blob, dst: torch.Tensor, stream=None) -> torch.Tensor:
    dtype = _check_tensor(dst, wide_ok=True)
    rc = _lib.neuzip_decompress(blob.handle, ctypes.c_void_p(dst.data_ptr()), dst.numel(), dtype,
                                _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_decompress")
    return dst


def neuzip_decompress_sequence(blobs, scratch: torch.Tensor, stream=None):
    """Decompresses the blobs in order into the one scratch tensor; returns, per blob, the index of its
    first element in the scratch (neighbouring blobs that fit together share the space and a launch)."""
    dtype = _check_tensor(scratch, wide_ok=True)
    arr = (ctypes.c_void_p * len(blobs))(*[b.handle.value for b in blobs])
    offsets = (ctypes.c_uint64 * len(blobs))()
    # the library counts the scratch, and the offsets, in 16-bit words
    rc = _lib.neuzip_decompress_sequence(arr, len(blobs), ctypes.c_void_p(scratch.data_ptr()),
                                         scratch.numel() * (2 if dtype == F32 else 1), offsets, _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_decompress_sequence")
    return [int(v) // (2 if dtype == F32 else 1) for v in offsets]


def neuzip_decompress_batch(blobs, dsts, stream=None) -> None:
    if len(blobs) != len(dsts) or any(b.elems != d.numel() or b.dtype != _check_tensor(d, wide_ok=True)
                                      for b, d in zip(blobs, dsts)):
        raise ValueError("one destination of matching size and element type per blob")
    arr = (ctypes.c_void_p * len(blobs))(*[b.handle.value for b in blobs])
    ptrs = (ctypes.c_void_p * len(dsts))(*[d.data_ptr() for d in dsts])
    rc = _lib.neuzip_decompress_batch(arr, ptrs, len(blobs), _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_decompress_batch")


def neuzip_linear(weight: Blob, out_features: int, in_features: int, x: torch.Tensor, bias: torch.Tensor = None,
                  y: torch.Tensor = None, stream=None) -> torch.Tensor:
    """y = x W_hat^T + bias with the weight taken straight from its compressed form (float32 result)."""
    _check_tensor(x)
    tokens = x.numel() // in_features if in_features else 0
    if x.numel() != tokens * in_features:
        raise ValueError("activations must be tokens x in_features")
    if y is None:
        y = torch.empty((tokens, out_features), dtype=torch.float32, device=x.device)
    if not (y.is_cuda and y.dtype == torch.float32 and y.is_contiguous() and y.numel() == tokens * out_features):
        raise TypeError("expected a contiguous float32 CUDA tensor of tokens x out_features")
    if bias is not None and not (bias.is_cuda and bias.dtype == torch.float32 and bias.is_contiguous()
                                 and bias.numel() == out_features):
        raise TypeError("expected a contiguous float32 CUDA bias of out_features")
    rc = _lib.neuzip_linear(weight.handle, out_features, in_features, ctypes.c_void_p(x.data_ptr()), tokens,
                            ctypes.c_void_p(bias.data_ptr() if bias is not None else None),
                            ctypes.c_void_p(y.data_ptr()), _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_linear")
    return y


def neuzip_linear_batch(weights, out_features, in_features: int, x: torch.Tensor, biases=None, ys=None,
                        stream=None):
    """y_i = x W_hat_i^T + bias_i for several compressed weights applied to the same activations, in one
    launch (at most 4 weights).  Returns the list of float32 results."""
    _check_tensor(x)
    count = len(weights)
    if len(out_features) != count or (biases is not None and len(biases) != count) or \
            (ys is not None and len(ys) != count):
        raise ValueError("weights, out_features, biases and ys must have one entry per weight")
    tokens = x.numel() // in_features if in_features else 0
    if x.numel() != tokens * in_features:
        raise ValueError("activations must be tokens x in_features")
    if ys is None:
        ys = [torch.empty((tokens, o), dtype=torch.float32, device=x.device) for o in out_features]
    for y, o in zip(ys, out_features):
        if not (y.is_cuda and y.dtype == torch.float32 and y.is_contiguous() and y.numel() == tokens * o):
            raise TypeError("expected contiguous float32 CUDA tensors of tokens x out_features")
    if biases is not None:
        for bias, o in zip(biases, out_features):
            if bias is not None and not (bias.is_cuda and bias.dtype == torch.float32 and bias.is_contiguous()
                                         and bias.numel() == o):
                raise TypeError("expected contiguous float32 CUDA biases of out_features")
    arr = (ctypes.c_void_p * count)(*[w.handle.value for w in weights])
    outs = (ctypes.c_uint64 * count)(*[int(o) for o in out_features])
    yp = (ctypes.c_void_p * count)(*[y.data_ptr() for y in ys])
    bp = None
    if biases is not None:
        bp = (ctypes.c_void_p * count)(*[(b.data_ptr() if b is not None else None) for b in biases])
    rc = _lib.neuzip_linear_batch(arr, outs, count, in_features, ctypes.c_void_p(x.data_ptr()), tokens, bp, yp,
                                  _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_linear_batch")
    return ys


def neuzip_free(blob: Blob) -> None:
    blob.free()


def neuzip_compressed_bytes(blob: Blob) -> int:
    return blob.compressed_bytes


def neuzip_export(blob: Blob, stream=None) -> np.ndarray:
    size = ctypes.c_uint64(0)
    rc = _lib.neuzip_export(blob.handle, None, 0, ctypes.byref(size), _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_export(size)")
    buf = np.empty(size.value, np.uint8)
    rc = _lib.neuzip_export(blob.handle, buf.ctypes.data_as(ctypes.c_void_p), buf.size, ctypes.byref(size),
                            _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_export")
    return buf


def neuzip_import(container: np.ndarray, stream=None) -> Blob:
    container = np.ascontiguousarray(container, dtype=np.uint8)
    handle = ctypes.c_void_p(None)
    rc = _lib.neuzip_import(container.ctypes.data_as(ctypes.c_void_p), container.size, _stream_handle(stream),
                            ctypes.byref(handle))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_import")
    return Blob(handle.value)


def neuzip_histogram(blob: Blob) -> np.ndarray:
    out = np.zeros(256, np.uint32)
    rc = _lib.neuzip_histogram(blob.handle, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_histogram")
    return out


def neuzip_frequencies(blob: Blob) -> np.ndarray:
    out = np.zeros(256, np.uint16)
    rc = _lib.neuzip_frequencies(blob.handle, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_frequencies")
    return out


def neuzip_stream_probe(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """Reads all of src and overwrites all of dst the way the decoder moves its bytes (a timing aid)."""
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise TypeError("expected contiguous CUDA tensors")
    rc = _lib.neuzip_stream_probe(ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                                  ctypes.c_void_p(dst.data_ptr()), dst.numel() * dst.element_size(), _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_stream_probe")


def neuzip_check(blob: Blob, stream=None) -> None:
    rc = _lib.neuzip_check(blob.handle, _stream_handle(stream))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_check")


def neuzip_workspace_bytes() -> int:
    return int(_lib.neuzip_workspace_bytes())


def neuzip_set_workspace_limit(slot_bytes: int) -> None:
    """Limit on the encoder's run slots in bytes (0: the default); larger tensors are compressed in tiles."""
    rc = _lib.neuzip_set_workspace_limit(int(slot_bytes))
    if rc != OK:
        raise NeuzipError(rc, "neuzip_set_workspace_limit")


def neuzip_release_workspace() -> None:
    rc = _lib.neuzip_release_workspace()
    if rc != OK:
        raise NeuzipError(rc, "neuzip_release_workspace")
