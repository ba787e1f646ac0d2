"""MI355X-native batch-1 SpMV over EC-CSR (block extraction + delta-compressed storage).

`binding` mirrors the C ABI of libecspmv.so one to one; `device` adds the few lines that let
PyTorch own the device buffers and streams.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    EcspmvError, Matrix, CsrMatrix, make_opts, ecspmv_build_dense, ecspmv_build_csr,
    ecspmv_build_dense_f32, ecspmv_build_csr_f32,
    ecspmv_csr_build_dense, ecspmv_stream_read, ecspmv_stream_read_sliced, ecspmv_empty_launch,
    ecspmv_run_batch, Batch,
)
