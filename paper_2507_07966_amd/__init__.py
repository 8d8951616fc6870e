"""Prefix-shared GRPO prefill attention for MI355X (gfx950).

`workloads` (seeded synthetic inputs) is plain numpy.  Everything else is the thin
ctypes binding over the C-ABI library built from csrc/; it is imported on first
use and raises if the library has not been built.
"""
from . import workloads  # noqa: F401

_BINDING_NAMES = ("PrefixAttnPlan", "PrefixAttnError", "prefix_attn_plan", "prefix_attn_forward", "prefix_attn_forward_static",
                  "prefix_attn_forward_timed", "STATIC_SCRATCH_BYTES",
                  "prefix_attn_lse", "prefix_attn_destroy", "prefix_attn_status_string",
                  "prefix_attn_backward", "prefix_attn_backward_timed", "prefix_attn_forward_partial",
                  "prefix_attn_merge_partials", "token_logprob_workspace", "token_logprob_forward",
                  "grpo_group_advantages",
                  "library_path", "load_library")


def __getattr__(name):
    if name == "binding" or name in _BINDING_NAMES:
        import importlib
        mod = importlib.import_module(".binding", __name__)
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError(name)
