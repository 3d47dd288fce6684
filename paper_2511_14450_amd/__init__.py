"""MI355X-native forward pass of one pipeline stage of decoder blocks.

The work is done by the HIP library `libhyp_stage.so` (C ABI in
include/hyp_stage.h); this package only marshals arguments.  Importing the
package does not load the library; the first call does, and fails loudly if it
has not been built (python -m paper_2511_14450_amd.build).
"""
from .binding import (  # noqa: F401
    HypError, LayerWeights, Stage, StageConfig, library_path, load_library,
    stage_context_len, stage_create, stage_decode_step, stage_decode_step_noalloc, stage_destroy, stage_export_kv,
    stage_last_error, stage_prefill, stage_set_page_table, stage_profile, stage_profile_read, stage_uses_mfma,
    stage_workspace_bytes, KERNEL_CLASSES, stage_config, hyp_measure_mfma_ceiling,
    hyp_measure_hbm_read_ceiling, hypsplit_dp, hypsched_rt, hypsched_simulate,
)


def __getattr__(name):
    # the chain module is also a program (python -m paper_2511_14450_amd.chain): load it on demand
    if name == "StageChain":
        from .chain import StageChain
        return StageChain
    raise AttributeError(name)
