"""MI355X-native draft verification for speculative decoding (block / token / greedy).

The work is done by HIP kernels in ``csrc/`` behind the C ABI of ``include/specverify.h``;
this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    SpecVerifyError, alloc_workspace, load, spec_verify_block, spec_verify_greedy,
    spec_verify_ex, spec_verify_ex_noalloc, spec_verify_probs, spec_verify_token, spec_verify_workspace_bytes, spec_verify_workspace_check,
    spec_verify_workspace_init, spec_verify_debug_config, spec_verify_debug_last_kernel, spec_verify_debug_profile,
    spec_verify_debug_copy, spec_verify_debug_stream_probe, spec_sample_tokens, status_string,
)
