"""MI355X-native quantized layer step of Coded Deep Learning (arxiv 2501.09849).

The work is done by hand-written HIP kernels for gfx950 behind the C library
declared in include/cdl.h; `binding` marshals arguments to it, nothing more.
"""
from .binding import (  # noqa: F401
    CdlError, QParams, lib_path, load,
    quantize_workspace_bytes, qgemm_fwd_workspace_bytes, qgemm_bwd_workspace_bytes,
    cdl_quantize_fwd, cdl_quantize_fwd_static, static_scratch_bytes, cdl_quantize_bwd, cdl_marginal_entropy, cdl_qgemm_fwd, cdl_qgemm_bwd,
    qgemm_fwd_offset_workspace_bytes, cdl_index_offset, cdl_qgemm_fwd_offset, cdl_qgemm_bwd_offset, cdl_qgemm_bwd_quantize_bwd,
    qconv_fwd_workspace_bytes, cdl_qconv_fwd, cdl_qgemm_fwd_quantize, qconv_bwd_weights_workspace_bytes, cdl_qconv_bwd_weights,
    qconv_bwd_activations_workspace_bytes, cdl_qconv_bwd_activations,
    cdl_quantize_draw, cdl_entropy_bwd, huffman_workspace_bytes, cdl_huffman_bits,
    cdl_profile_enable, cdl_profile_collect, cdl_profile_only, cdl_probe_mfma_int8, EXPORTS,
)
