"""HBM-resident parameter server pull/push for one MI355X: Python binding of libhps.so.

The binding marshals arguments only; every step of the path runs in the HIP
kernels behind the C ABI (include/hps.h); the host-memory cache behind the table
(include/hps_mem.h) is native host code.  torch supplies device memory and the
current stream.
"""
from .binding import (  # noqa: F401
    HpsError,
    HpsTable,
    MemStats,
    MemTier,
    Optimizer,
    Stats,
    lib,
    probe_random_rows,
    ADAGRAD_ROWWISE,
    ADAGRAD_ELEMENTWISE,
    ROWS_F32,
    ROWS_BF16,
    ROWS_F32_WIDE,
    OK, EINVAL, EFULL, ERESERVED, ESTATE, EDEVICE, ENOMEM,
    EXPORTS,
    STAGES,
)
