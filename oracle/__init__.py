"""CPU oracle (test infrastructure only) for the SendRecv / AlltoAll(v) path.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It imports nothing from the GPU library.
"""
from .oracle import (  # noqa: F401
    build,
    alltoallv,
    alltoall,
    sendrecv,
    sendrecv_staged,
    moe_pack,
    moe_pack_dedup,
    moe_unpack,
    moe_exchange_layout,
    OracleError,
)
