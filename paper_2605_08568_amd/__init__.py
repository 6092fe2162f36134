"""MI355X (gfx950) routed low-rank linear layer: thin Python binding over the C-ABI library libparse.so.

Every step of the path runs in the library's HIP kernels; this package only marshals arguments
(PyTorch supplies device memory and streams).  Importing it without a built library raises."""
from .binding import (  # noqa: F401
    PARSE_BF16, PARSE_DECODE, PARSE_F32, PARSE_MFMA16, PARSE_PREFILL, PARSE_ROWMAJOR,
    Cache, Layer, ParseError, Patterns, bf16_from_bits, bf16_to_bits, bucket_patterns,
    check_offsets, check_subset, layer_to_mfma16, lib, lowrank_decode_multi, lowrank_decode_multi_workspace_bytes, lowrank_decode_static,
    lowrank_prefill_multi, lowrank_prefill_multi_workspace_bytes,
    lowrank_forward, lowrank_workspace_bytes,
    pack_experts, pack_new_entries, pack_patterns, pack_ranks, rankmajor_left_factor, pool, route, route_ranks, router_grad, route_workspace_bytes, status_string, version,
    PARSE_SCHED_AUTO, PARSE_SCHED_FUSED, PARSE_SCHED_TILES, PARSE_SCHED_PLANNED, prefill_plan, prefill_plan_bytes, bucket_and_plan,
    lowrank_prefill_planned, lowrank_prefill_planned_workspace_bytes,
    probe_mfma_bf16, probe_read, probe_copy,
    decode_plan, lowrank_decode_planned, lowrank_decode_planned_workspace_bytes,
)
