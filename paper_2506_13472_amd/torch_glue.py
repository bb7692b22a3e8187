"""PyTorch is used for device memory and streams only: allocate y and the
workspace, hand raw pointers and the current stream to the C ABI."""
from __future__ import annotations

import torch

from . import binding as B


def current_stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def alloc_workspace(p: B.Packed, M: int) -> torch.Tensor:
    n = B.rosaq_workspace_bytes(p, M)
    return torch.empty(n, dtype=torch.uint8, device="cuda")


def linear(p: B.Packed, x: torch.Tensor, y: torch.Tensor | None = None,
           ws: torch.Tensor | None = None) -> torch.Tensor:
    """y = rosaq_linear*(p, x) on the current stream.  x: fp16 [M, D] on the GPU
    (row stride may exceed D)."""
    if not x.is_cuda or x.dtype != torch.float16 or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-D fp16 CUDA tensor with unit column stride")
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, p.N), dtype=torch.float16, device=x.device)
    if ws is None:
        ws = alloc_workspace(p, M)
    fn = B.rosaq_linear_headwise if p.q_mode == B.Q_HEADWISE else B.rosaq_linear
    fn(p, x.data_ptr(), M, x.stride(0), y.data_ptr(), y.stride(0), ws.data_ptr(), ws.numel(),
       current_stream_ptr())
    return y


def linear_batch(layers, x: torch.Tensor, ys=None, ws: torch.Tensor | None = None):
    """[y_i] = rosaq_linear_batch(layers, x): layers share x and the rotation."""
    M = x.shape[0]
    if ys is None:
        ys = [torch.empty((M, p.N), dtype=torch.float16, device=x.device) for p in layers]
    if ws is None:
        ws = alloc_workspace(layers[0], M)
    args = B.BatchArgs(layers, [y.data_ptr() for y in ys], [y.stride(0) for y in ys])
    B.rosaq_linear_batch(args, x.data_ptr(), M, x.stride(0), ws.data_ptr(), ws.numel(),
                         current_stream_ptr())
    return ys
