"""MI355X-native embedding hot path of a Slipstream training step.

`workload` draws the seeded synthetic inputs.  `binding` (imported on first
use of any `ss_*` name) loads libslipstream.so, the HIP library behind the
C ABI declared in include/slipstream.h, and raises if it is missing: there
is no CPU fallback.
"""
from . import workload  # noqa: F401

_BINDING_NAMES = (
    "Tables", "ss_embbag_forward", "ss_embbag_backward_update",
    "ss_detect_stale", "ss_filter_batch", "ss_filter_batch_workspace_bytes",
    "ss_backward_workspace_bytes", "ss_last_error", "SlipstreamError",
    "ss_profile_enable", "ss_profile_report", "HotState",
    "ss_embbag_backward_prepare", "ss_embbag_backward_apply",
    "ss_embbag_forward_grouped", "ss_sample_drop", "ss_drop_stats",
    "ss_count_accesses", "ss_select_hot_workspace_bytes", "ss_select_hot_ratio",
    "ss_select_hot_top", "AccessCounters", "ss_layernorm_forward",
    "ss_layernorm_backward", "ss_layernorm_backward_workspace_bytes",
    "ss_embbag_forward_ln", "ss_embbag_ln_backward",
    "ss_embbag_backward_update_noalloc", "ss_filter_batch_split", "ss_check_enable",
    "ss_check_indices", "ss_step_plan_for", "ss_step_create", "ss_step_destroy",
    "ss_step_room", "ss_step_submit", "ss_step_forward", "ss_step_backward", "ss_step_flush",
    "EmbeddingStep", "PipelinedStep", "lib_path",
)


def __getattr__(name):
    if name in _BINDING_NAMES or name in ("binding", "step"):
        import importlib
        if name in ("step", "EmbeddingStep", "PipelinedStep"):
            mod = importlib.import_module(".step", __name__)
            return mod if name == "step" else getattr(mod, name)
        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError(name)
