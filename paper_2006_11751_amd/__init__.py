"""MI355X-native policy-worker step (paper Sec. 3.1): HIP library + thin binding.

`workloads` (numpy only) may be imported on its own; the binding names
(`sf_policy_create`, `sf_policy_step`, `sf_policy_destroy`, `sf_last_error`,
`Policy`) are resolved lazily and raise if the HIP library has not been built.
"""

_BINDING_NAMES = ("sf_policy_create", "sf_policy_step", "sf_policy_step_indexed", "sf_policy_update_weights", "sf_policy_destroy", "sf_appo_loss",
                  "sf_appo_loss_workspace_bytes", "appo_loss",
                  "sf_last_error", "sf_pipeline_create", "sf_pipeline_submit", "sf_pipeline_wait",
                  "sf_pipeline_destroy", "Policy", "Pipeline", "SfError", "load_library",
                  "build_library", "library_path")


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
