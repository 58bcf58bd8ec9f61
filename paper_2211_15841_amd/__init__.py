"""MI355X-native dropless-MoE (dMoE) expert layer: thin Python binding over the C-ABI library libdmoe.so.

Every step of the layer runs in the hand-written HIP kernels of csrc/; Python only marshals arguments and
uses torch for device memory and the stream handle.  There is no CPU or eager fallback: importing the
binding without the built library raises.
"""
from .binding import (  # noqa: F401
    DMoEConfig, DMoETopology, Workspace, load_library, dmoe_sizes, dmoe_topology_bind, dmoe_topology, dmoe_topology_static,
    dmoe_forward, dmoe_backward, dmoe_backward_accumulate, dmoe_topology_counts_host, dmoe_set_stage_events, dmoe_set_tile_mode, dmoe_last_error,
    STAGE_NAMES, DMoEError, BlockSparse, dmoe_bsmm_sizes, dmoe_bsmm_topology, dmoe_bsmm,
    OP_SDD, OP_DSD, OP_SDDT, OP_DSTD, OP_DSDT, OP_DDTS, OP_DDS, OP_SDTD, OP_SDTDT, OP_DSTDT, OP_DDST, OP_DDTST, dmoe_probe_mfma_tflops, dmoe_probe_mfma_sustained,
)
