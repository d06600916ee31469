"""MI355X-native Evoformer gated axial attention with pair bias (FastFold, arXiv 2203.00854).

The product is the HIP library libff.so behind the C ABI of include/ff.h; this package
holds its sources (csrc/), the build step, a thin ctypes binding and the seeded input
generators used by the tests and the benchmark.
"""
from .binding import (  # noqa: F401
    FF_BF16, FF_F32, FF_MSA_COL, FF_MSA_ROW, FF_TRI_END, FF_TRI_START, AttnDesc, AttnWeights, FFError, TriMulDesc, TriMulWeights, GlobalDesc, GlobalWeights, CoreDesc, ff_attention_core_backward,
    ff_attention_core_backward_workspace_bytes, core_to_device, ff_global_column_attention,
    ff_global_column_attention_workspace_bytes, global_to_device, ff_triangle_multiplication,
    ff_triangle_multiplication_workspace_bytes, trimul_to_device,
    ff_attention_chunked, ff_attention_last_path, ff_attention_path, ff_profile_collect, ff_profile_enable, ff_attention_workspace_bytes, ff_gated_attention, ff_gated_attention_residual, ff_gated_attention_static, ff_layernorm, ff_probe_copy, ff_probe_mfma, ff_probe_valu, ff_static_scratch_bytes,
    last_error, lib, make_desc, make_weights, to_device,
)
