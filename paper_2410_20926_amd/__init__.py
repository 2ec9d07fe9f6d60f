"""MI355X-native Tensorized Attention (arXiv 2410.20926): thin Python binding over
the C-ABI library libtensattn.so.  Importing this package does not load the
library; the first call does, and fails loudly if it has not been built."""
from .tensattn import (  # noqa: F401
    TA_BF16, TA_F32, TA_VIN_KV, TA_VIN_O, Plan, TaDesc, TaError, library_path, load_library,
    ta_axis_attn_backward, ta_axis_attn_forward, ta_axis_pair_attn_forward, ta_copy_bytes, ta_stream_mix, ta_stream_slabs, ta_multihop_backward,
    ta_multihop_forward, ta_multihop_forward_static, TA_STATIC_WORKSPACE_BYTES, ta_plan_create, ta_rope_apply, ta_version, pack_axis_mask,
)
