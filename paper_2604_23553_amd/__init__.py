"""cfpp: MI355X-native single-token decode of GPT-NeoX / Pythia decoder blocks.

The product is the C-ABI HIP library `libcfpp.so` (see include/cfpp.h); this
package is its thin ctypes binding.  Every step of the decode path runs in the
library's kernels; PyTorch is used by callers only for device memory and streams.
"""
from .binding import (  # noqa: F401
    CfppError, Config, lib, library_path, profile_build,
    cfpp_validate_config, cfpp_packed_layer_bytes, cfpp_kv_layer_bytes, cfpp_workspace_bytes,
    cfpp_algorithmic_bytes, cfpp_pack_layer, cfpp_kv_import, cfpp_kv_export,
    cfpp_create, cfpp_destroy, cfpp_set_option, cfpp_get_option,
    cfpp_block_decode, cfpp_stack_decode, cfpp_stack_prefill, cfpp_prefill_scratch_bytes, cfpp_stack_prefill_gemm, cfpp_stack_capture, cfpp_stack_replay,
    cfpp_block_decode_static, cfpp_device_error, cfpp_debug_read, cfpp_stream_read, cfpp_stream_copy,
    Lm, cfpp_lm_embed, cfpp_lm_next, cfpp_generate_capture,
    OPT_MODE, OPT_GRID, OPT_THREADS, OPT_PROFILE_SKIP, OPT_EPOCH_LIMIT, MODE_AUTO,
)
