"""MI355X-native Swimba token mixer: HIP kernels behind a C ABI (libswimba.so)
and a thin binding with the same names.  `synth` holds the seeded input
recipe.  Nothing here falls back to the CPU."""

_BINDING_NAMES = (
    "swimba_mixer_fwd", "swimba_expert_proj", "swimba_expert_proj_workspace_bytes",
    "swimba_expert_proj_selected", "swimba_mixer_fwd_selected", "swimba_mixer_fwd_proj",
    "swimba_mixer_proj_workspace_bytes", "swimba_router_linear", "swimba_mixer_fwd_xe", "swimba_mixer_fwd_xe_selected", "swimba_expert_proj_x_selected", "swimba_expert_proj_x_workspace_bytes",
    "swimba_mixer_fwd_xe_proj", "swimba_mixer_xe_proj_workspace_bytes", "swimba_mixer_xe_selected_workspace_bytes", "swimba_mixer_xe_workspace_bytes", "swimba_separated_fwd", "swimba_separated_workspace_bytes", "swimba_step", "swimba_step_multi", "swimba_step_multi_workspace_bytes", "swimba_step_workspace_bytes", "swimba_router_topk", "swimba_mixer_workspace_bytes",
    "swimba_mixer_workspace_layout", "swimba_stage_router", "swimba_stage_cumsum",
    "swimba_stage_mix", "swimba_stage_chunk_state", "swimba_stage_state_scan", "swimba_stage_output",
    "swimba_stage_prep", "swimba_stage_mix_chunk", "swimba_stage_tables", "PATH_SINGLE_PASS_CHUNK_MIX", "PATH_SINGLE_PASS_HEAD", "PATH_SINGLE_PASS_HEAD_CHUNK_MIX", "swimba_stage_pass", "swimba_stage_pass64", "swimba_stage_boundary_states", "swimba_stage_pass64_split", "swimba_pass_segments", "PATH_SINGLE_PASS_HEAD_SPLIT", "PATH_SINGLE_PASS_HEAD_SPLIT_CHUNK_MIX", "swimba_stage_chunk_state_tiles", "swimba_stage_output_carry", "PATH_STAGED_SHORT", "swimba_prefill_path", "swimba_step_static",
    "PATH_GENERIC", "PATH_STAGED", "PATH_SINGLE_PASS",
    "swimba_probe_copy", "swimba_probe_mfma", "alloc_workspace", "workspace_views", "dims_of",
    "make_dims", "SwimbaError", "library_loaded",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
