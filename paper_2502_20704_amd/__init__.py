"""MI355X-native candidate verification for Fuzzy Speculative Decoding.

``paper_2502_20704_amd.fsd_verify_chain`` / ``fsd_verify_tree`` / ``sd_verify_chain`` /
``rfsd_verify_chain`` marshal
torch tensors into the C ABI of ``libfsd.so`` (see ``include/fsd.h``); every step of the method
runs in the HIP kernels.  ``paper_2502_20704_amd.synth`` makes the seeded synthetic inputs.
"""
from .binding import (  # noqa: F401
    DIV_JS, DIV_KL, DIV_TV, F32, BF16, GREEDY, SAMPLE,
    ROW_BAD_PARENT, ROW_BAD_TOKEN, ROW_INTERNAL, ROW_NONFINITE, ROW_TOO_DEEP,
    FsdError, fsd_verify_chain, fsd_verify_chain_static, STATIC_SCRATCH_BYTES, fsd_verify_chain_warped, fsd_verify_tree, fsd_verify_tree_warped, fsd_workspace_bytes, library, sd_verify_chain, sd_verify_tree, rfsd_verify_chain, fsd_calibrate_threshold,
    profile_enable, profile_collect, debug_set_spin_limit, debug_set_shape, debug_warp_thresholds, debug_set_js_floor, debug_set_exact_js, debug_set_self_clear,
)
