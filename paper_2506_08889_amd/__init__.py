"""MI355X-native decode hot path of SeerAttention-R: AttnGate block selection and
block-sparse flash-decoding, as hand-written gfx950 HIP kernels behind a small C ABI
(``include/seer.h``).  This package is only the thin Python binding: argument marshalling,
no arithmetic.  PyTorch is used for device memory and streams.
"""
from .api import (  # noqa: F401
    HINT_RAGGED_LISTS, NOALLOC_SCRATCH_BYTES, SELECT_THRESHOLD, SELECT_TOPK, SELECT_TOPP, KERNEL_CLASSES, SeerError,
    attn_ground_truth,
    attn_ground_truth_workspace_bytes, decode_plan, dense_decode, decode_workspace_bytes,
    gate_q, gate_select, gate_select_q, gate_workspace_bytes, get_knob, hbm_read_probe, kc_update, lib_path, load_library, profile_durations, profile_enable, profile_read,
    profile_reset, set_knob, sparse_decode, sparse_decode_multi, sparse_decode_noalloc, version,
)
