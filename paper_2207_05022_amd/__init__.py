"""Python binding of libsti (MI355X / gfx950 shard decode + encoder layer).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libsti.so``.  Importing this package fails loudly when the library has not
been built (``python paper_2207_05022_amd/build.py``); there is no fallback.
"""
from .binding import (  # noqa: F401
    STI_F32, STI_F16, STI_BF16, STI_PREC_F32, STI_PREC_F16_MFMA,
    StiError, StiDims, StiShard, StiLayerParams, lib, status_string,
    sti_decode_workspace_bytes, sti_decode_shards, sti_workspace_bytes,
    sti_layer_forward, sti_model_forward, sti_layer_forward_masked, sti_model_forward_masked, sti_profile_begin, sti_profile_end, sti_pipeline_staging_bytes, sti_model_workspace_bytes, sti_plan_submodel, sti_plan_bitwidths, sti_quantize_workspace_bytes, sti_quantize_layer, StiQuantStats, StiPipeline, StiPipelineStats, make_store, shard_array, sti_layer_forward_static,
    sti_working_buffer_bytes, sti_working_buffer_offset, sti_decode_working_buffer,
)
