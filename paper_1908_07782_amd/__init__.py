"""Segmented-gossip aggregation round on one MI355X: thin Python binding of libcombo.

The functions below have the names and argument order of the C ABI (include/combo.h)
and only marshal arguments: torch tensors supply device memory and the stream, every
step of the round runs in the library's HIP kernels.  There is no CPU fallback: if the
shared library has not been built, importing the binding's functions raises.
"""
from . import workloads  # noqa: F401
from .arena import GossipArena  # noqa: F401
from .binding import (ComboError, get_tune, round_kernel_kind, lib, local_sgd_then_gossip, make_peer_table,
                      make_peer_table_pooled, peer_in_degree, make_peer_table_dynamic,
                      segment_gossip_round_dynamic, aggregation_divergence,
                      aggregation_divergence_workspace, local_sgd_steps_then_gossip,
                      tiled_cols, tiled_elems, pack_tiled, unpack_tiled,
                      segment_gossip_round_tiled, local_sgd_steps_then_gossip_tiled,
                      aggregation_divergence_tiled, round_hashed, aggregation_divergence_noalloc, round_relayout, bandwidth_probe, PROBE_COPY, PROBE_READ, PROBE_WRITE,
                      PROBE_ROW_CHUNKS, PROBE_TILES, PROBE_MULTI_READ, PROBE_LDS_READ,  # noqa: F401
                      segment_gossip_round, strerror, tune, TUNE_FUSED_MODE, TUNE_TILE_COLS,
                      TUNE_XCD_SWIZZLE, TUNE_KERNEL, TUNE_SLAB_COLS, TUNE_SLAB_ORDER, TUNE_SLAB_THREADS, TUNE_SLAB_LDS_FLOOR, LIB_PATH)
