"""A linear layer whose weight is held compressed, and the layer-by-layer training step of Alg. 1.

Orchestration only: every codec step is a call into the HIP library (binding.py); the dense
products of the backward pass are torch's (a library GEMM is the right tool for a training batch).

Alg. 1, forward loop: for each layer the weight is decompressed into temporary space just before
it is used (Sec. 2.2, Eq. (3)); here a decoding batch of up to 64 tokens goes through the fused
kernel instead, which never writes the weight.  Backward loop: the weight is decompressed again,
the gradients of the layer are formed, the optimiser step is applied at once and the weight is
compressed again, so that neither the uncompressed model nor the full set of gradients ever exists.

Biases are not compressed (Sec. 2.1 and 2.2 treat weight matrices only): they are plain float32
tensors of the caller's, and their addition and their own SGD step below are ordinary torch
arithmetic outside the codec's path.
"""
import torch

from . import binding as nz


class CompressedLinear:
    """y = x W^T + b with W (out_features x in_features, bf16) stored as a lossless blob."""

    def __init__(self, weight: torch.Tensor, bias: torch.Tensor = None, guard: int = 8):
        if weight.dim() != 2 or weight.dtype != torch.bfloat16:
            raise TypeError("weight: a 2-d bf16 tensor")
        self.out_features, self.in_features = weight.shape
        (self.blob,) = nz.neuzip_compress_guarded([weight.contiguous()], 7, guard)
        self.bias = None if bias is None else bias.to(torch.float32).contiguous()

    def weight_into(self, space: torch.Tensor) -> torch.Tensor:
        """W_hat <- decompress(c) into the caller's temporary space; returns it shaped as the matrix."""
        flat = space.view(-1)[: self.out_features * self.in_features]
        nz.neuzip_decompress(self.blob, flat)
        return flat.view(self.out_features, self.in_features)

    def forward(self, x: torch.Tensor, space: torch.Tensor) -> torch.Tensor:
        """x: tokens x in_features, bf16.  Returns float32 tokens x out_features."""
        tokens = x.shape[0]
        if tokens <= 64 and self.in_features % 128 == 0:
            return nz.neuzip_linear(self.blob, self.out_features, self.in_features, x.contiguous(), self.bias)
        y = torch.matmul(x, self.weight_into(space).t()).float()
        return y if self.bias is None else y + self.bias

    def backward_and_update(self, x: torch.Tensor, grad_y: torch.Tensor, lr: float, space: torch.Tensor,
                            grad_space: torch.Tensor):
        """The layer's part of the backward loop.  x: the input the forward pass saw (bf16), grad_y: the
        gradient of the loss with respect to the layer's output (bf16), both tokens x features.
        Returns (grad_x, rebuilt flag); the blob holds the updated weight afterwards and `grad_space`
        the weight gradient that was applied (bf16); what `space` holds is unspecified."""
        w_hat = self.weight_into(space)                                   # the second decompression
        grad_x = torch.matmul(grad_y, w_hat)                              # tokens x in_features
        n = self.out_features * self.in_features
        grad_w = grad_space.view(-1)[:n].view(self.out_features, self.in_features)
        torch.matmul(grad_y.t(), x, out=grad_w)                           # out_features x in_features, bf16
        if self.bias is not None:
            self.bias -= lr * grad_y.float().sum(dim=0)
        # `space` still holds W_hat from the decompression above: the step and the coding are one pass,
        # and nobody needs the new weight uncompressed
        (rebuilt,) = nz.neuzip_update([self.blob], [grad_w.view(-1)], [space.view(-1)[:n]], lr, weights_ready=2)
        return grad_x, rebuilt


def training_step(layers, x: torch.Tensor, target: torch.Tensor, lr: float, space: torch.Tensor,
                  grad_space: torch.Tensor, observer=None):
    """One step of Alg. 1 on a stack of CompressedLinear layers with ReLU between them and a squared
    error loss: forward layer by layer keeping the layer inputs, then backward in reverse order, each
    weight updated and recompressed as soon as its gradient exists.  Returns (loss, rebuilt flags).
    observer(i, layer_input, grad_y, grad_w), if given, is called right after layer i's update."""
    inputs, h = [], x
    for i, layer in enumerate(layers):
        inputs.append(h)
        y = layer.forward(h, space)
        h = (torch.relu(y) if i + 1 < len(layers) else y).to(torch.bfloat16)
    diff = h.float() - target.float()
    loss = 0.5 * (diff * diff).sum().item()
    grad = diff.to(torch.bfloat16)
    flags = [0] * len(layers)
    for i in reversed(range(len(layers))):
        if i + 1 < len(layers):
            grad = grad * (inputs[i + 1] > 0)                            # ReLU of layer i fed layer i + 1
        grad_y = grad.contiguous()
        grad, flags[i] = layers[i].backward_and_update(inputs[i], grad_y, lr, space, grad_space)
        if observer is not None:
            n = layers[i].out_features * layers[i].in_features
            observer(i, inputs[i], grad_y, grad_space.view(-1)[:n].view(layers[i].out_features, layers[i].in_features))
    return loss, flags
