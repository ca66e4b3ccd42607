"""MI355X-native P2P data movement behind SendRecv and AlltoAll(v).

A thin ctypes binding over ``libvccl.so`` (hand-written HIP kernels and a
copy-engine proxy behind a C boundary, see ``include/vccl.h``).  The binding
only marshals arguments: every step of the path runs inside the library.
There is no CPU fallback - if the library has not been built, importing the
binding's functions raises.
"""
import os as _os

# Ask the HIP runtime to carry out stream wait-value operations in the command
# processor instead of with a helper kernel, so that the copy-engine path dispatches
# nothing at all (see VCCL_MODE_CE in include/vccl.h).  The runtime reads the variable
# when it starts, i.e. at the process's first HIP call: import this package before
# anything touches the GPU.  An explicit setting of the variable is left alone.
_os.environ.setdefault("GPU_STREAMOPS_CP_WAIT", "1")

from .binding import (  # noqa: E402,F401
    MODE_CU, MODE_CE, MODE_CU_STAGED,
    VcclError,
    lib_path, load, pointer_array,
    vccl_init, vccl_finalize, vccl_last_error, vccl_set_option, vccl_get_option,
    vccl_sendrecv, vccl_sendrecv_staged_status, vccl_p2p_reginfo,
    vccl_p2p_export, vccl_p2p_connect, vccl_p2p_recv, vccl_p2p_send, vccl_p2p_record, vccl_p2p_abort, vccl_p2p_close,
    vccl_alltoall, vccl_alltoallv, vccl_plan_alltoallv,
    vccl_moe_pack, vccl_moe_pack_noalloc, vccl_moe_pack_per_rank, vccl_moe_dispatch_fused, vccl_moe_combine_fused, vccl_moe_unpack, vccl_moe_exchange_layout,
    vccl_fma_probe, vccl_fma_probe_clocks, vccl_device_wall_clock_khz, vccl_hbm_probe, vccl_proxy_stats, vccl_proxy_cpu_time, vccl_device_cu_count,
    vccl_monitor_create, vccl_monitor_destroy, vccl_monitor_post, vccl_monitor_complete,
    vccl_monitor_totals, vccl_proxy_monitor,
)
