"""MI355X-native expert-group side of one MoE layer (FinDEP hot path).

The work is done by hand-written HIP kernels in ``libmoe_ep.so`` behind the C ABI of
``include/moe_ep.h``; this package only marshals arguments.  There is no CPU fallback:
if the library has not been built, importing the binding raises.
"""
from .binding import (DEP_AASS, DEP_ASAS, DepConfig, DepModels, DepPrimitives, DepProblem, dep_layer_models,
                      dep_makespan, dep_replay, dep_search, dep_solve_r2, dep_tokens_per_expert, IO_DEVICE, IO_PINNED_HOST, ORDER_INTERLEAVED, ORDER_SHARED_FIRST, STAGES,
                      MoeEp, MoeEpConfig, MoeEpError, PipelineModel, choose_chunks, fit_linear, lib_path,
                      load_library, load_probe_library, pipeline_makespan, validate_config, validate_forward,
                      probe_device, routed_tile_rows, workspace_bytes, prepared_weight_bytes, forward_noalloc,
                      NOALLOC_SCRATCH_BYTES)

__all__ = ["MoeEp", "MoeEpConfig", "MoeEpError", "load_library", "load_probe_library", "lib_path", "validate_config",
           "validate_forward", "workspace_bytes", "prepared_weight_bytes", "ORDER_SHARED_FIRST", "ORDER_INTERLEAVED",
           "IO_DEVICE", "IO_PINNED_HOST", "STAGES", "PipelineModel", "fit_linear", "pipeline_makespan",
           "choose_chunks", "DepModels", "DepProblem", "DepConfig", "DepPrimitives", "DEP_ASAS", "DEP_AASS",
           "dep_layer_models", "dep_tokens_per_expert", "dep_replay", "dep_makespan", "dep_solve_r2",
           "dep_search", "routed_tile_rows", "probe_device", "forward_noalloc", "NOALLOC_SCRATCH_BYTES"]
