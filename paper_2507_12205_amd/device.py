"""PyTorch plumbing around the C ABI: device buffers and streams only, no arithmetic."""
from __future__ import annotations

import torch

from . import binding as B


def _stream_handle(stream=None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def upload(mat: B.Matrix, device="cuda:0", stream=None) -> torch.Tensor:
    """Allocate the device image with PyTorch, copy the EC-CSR image into it, return the buffer."""
    nbytes = mat.ecspmv_device_bytes()
    buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
    assert buf.data_ptr() % 256 == 0
    mat.ecspmv_upload(buf.data_ptr(), nbytes, _stream_handle(stream), keepalive=buf)
    return buf


def run(mat: B.Matrix, x: torch.Tensor, y: torch.Tensor, stream=None) -> torch.Tensor:
    """y = W x on the given (or current) stream; x, y are CUDA tensors of length n, m: FP16, or FP32 for a matrix
    built from FP32 values."""
    want = torch.float32 if mat.ecspmv_stats().value_bits == 32 else torch.float16
    assert x.dtype == want and y.dtype == want and x.is_cuda and y.is_cuda
    assert x.is_contiguous() and y.is_contiguous()
    mat.ecspmv_run(x.data_ptr(), y.data_ptr(), _stream_handle(stream))
    return y


def run_multi(mat: B.Matrix, X: torch.Tensor, Y: torch.Tensor, stream=None) -> torch.Tensor:
    """Y = W X for X of shape (n, nb), Y of shape (m, nb), row-major, nb in {1, 2, 4, 8}; FP16, or FP32 for a matrix
    built from FP32 values."""
    want = torch.float32 if mat.ecspmv_stats().value_bits == 32 else torch.float16
    assert X.dtype == want and Y.dtype == want and X.is_cuda and Y.is_cuda
    assert X.dim() == 2 and Y.dim() == 2 and X.shape[1] == Y.shape[1] and X.is_contiguous() and Y.is_contiguous()
    mat.ecspmv_run_multi(X.data_ptr(), Y.data_ptr(), int(X.shape[1]), _stream_handle(stream))
    return Y


def csr_upload(csr: B.CsrMatrix, device="cuda:0", stream=None) -> torch.Tensor:
    nbytes = csr.ecspmv_csr_device_bytes()
    buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
    csr.ecspmv_csr_upload(buf.data_ptr(), nbytes, _stream_handle(stream), keepalive=buf)
    return buf


def csr_run(csr: B.CsrMatrix, x: torch.Tensor, y: torch.Tensor, stream=None) -> torch.Tensor:
    assert x.dtype == torch.float16 and y.dtype == torch.float16 and x.is_cuda and y.is_cuda
    csr.ecspmv_csr_run(x.data_ptr(), y.data_ptr(), _stream_handle(stream))
    return y
