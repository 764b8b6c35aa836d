"""MI355X-native forward pass of one MoTE layer (Mixture of Ternary Experts, arXiv 2506.14435).

The product is libmote.so, a C-ABI library of hand-written HIP kernels for gfx950
(include/mote.h).  This package is its thin ctypes binding plus the in-tree build step.
"""
from .binding import (EXPORTS, KNOBS, ForwardGraph, LIB_PATH, STAGE_NAMES, TAP_FIELDS, MoteError, MoteLayer, alloc_taps,  # noqa: F401
                      load_library, mote_calib_copy, mote_event_pair_overhead, mote_block_forward, mote_layer_forward, mote_layer_forward_static, mote_pack_rtn, mote_pack_ternary,
                      mote_router_balance, mote_rtn_packed_bytes, mote_ste_linear_backward,
                      mote_packed_bytes, mote_router_topk, mote_stage_times, mote_stage_timing,
                      mote_tuning_set, mote_version)
