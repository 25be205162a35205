"""MI355X-native scoring + SubSample hot path of SPECS (arxiv 2506.15733).

The compute lives in libspecs_hip.so (hand-written HIP for gfx950 behind the C ABI of
include/specs.h). This package is argument marshalling only; there is no CPU fallback: every
entry point raises if the library has not been built.
"""
from .binding import (load_library, SpecsError, specs_workspace_bytes, specs_ctx_create, specs_ctx_destroy,
                      specs_ctx_status, specs_model_create, specs_model_destroy, specs_prefix_create,
                      specs_prefix_destroy, specs_prefill, specs_score_blocks, specs_score_blocks_static,
                      specs_score_target_and_reward, specs_commit_block,
                      specs_commit_block_dev, specs_select_and_switch, specs_path_counts,
                      specs_subsample, specs_strerror, specs_op_linear, specs_op_gate_up,
                      specs_op_lmhead_logprob, specs_op_attention, specs_op_qkv_rope, specs_ctx_profile, specs_ctx_profile_read,
                      ModelDescC, EXPORTED_SYMBOLS)
