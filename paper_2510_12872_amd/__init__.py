"""MI355X (gfx950) implementation of KVComm's cache-reuse hot path (arxiv 2510.12872).

The product is the C-ABI library libkvcomm.so declared in include/kvcomm.h; `binding`
marshals torch device tensors into its entry points.  Importing this package does
not load the library: that happens on the first call and fails loudly if it was not built
(there is no CPU fallback).
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    MAX_ANCHORS, MAX_BATCH, RULE_COSINE_SOFTMAX, RULE_L2_SOFTMAX, RULE_NEAREST, W_LAYER_HEAD_TOKEN, W_SEGMENT, W_TOKEN, KVCommError, Model,
    kvcomm_align_kv, kvcomm_align_kv_batch, kvcomm_align_kv_q8, kvcomm_align_kv_q8_batch, kvcomm_anchor_predict, kvcomm_anchor_predict_workspace, kvcomm_anchor_weights,
    kvcomm_anchor_weights_batch, kvcomm_anchor_weights_batch_workspace,
    kvcomm_anchor_weights_rule, kvcomm_anchor_weights_rule_workspace, kvcomm_anchor_weights_static,
    kvcomm_anchor_weights_static_capacity, kvcomm_anchor_weights_workspace,
    kvcomm_capture_offsets, kvcomm_quantize_deltas, kvcomm_suffix_attn, kvcomm_suffix_attn_confined, kvcomm_suffix_attn_workspace, kvcomm_weight_slots, library_path,
    load_library,
)
