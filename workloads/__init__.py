"""Seeded synthetic workloads: tensor shapes, value distributions and the
data-movement chains of the five benchmark configurations (plus the QKV projection that
stores through a virtual tensor).

This package holds *descriptions* only: random source tensors and, for each
configuration, the list of data-movement operators between the producer and the
consumer written as plain tuples.  It contains none of the method's arithmetic:
no index maps, no copies, no consumers.  Both the CPU oracle and the GPU path
read their inputs from here and nothing else is shared between them.
"""
from .inputs import (  # noqa: F401
    Workload,
    encode,
    c1_tiny_chain,
    c2_chain,
    c2_decode_attention,
    c3_oproj_gemm,
    c4_window_ln_linear,
    c5_moe_dispatch,
    qkv_proj_store,
    decode_segment,
    paged_decode_attention,
    moe_combine,
    qkv_store_chain,
    random_chain,
    rowsum_chain_large,
    CONFIGS,
)
