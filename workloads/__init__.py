"""Seeded synthetic inputs for the SendRecv / AlltoAll(v) data-movement path.

This package only manufactures input data (payload bytes, routing tables,
count/displacement layouts).  It contains none of the exchange or pack
arithmetic and is the one module both the CPU oracle's tests and the GPU
path's tests may import.
"""
from .generators import (  # noqa: F401
    MASTER_SEED,
    config_seed,
    splitmix64,
    payload_bytes,
    payload_words,
    normal_bf16_bits,
    zipf_topk_expert_ids,
    equal_layout,
    random_layout,
    ring_peers,
    pp_message_bytes,
)
