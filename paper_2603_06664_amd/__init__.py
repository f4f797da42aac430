"""MI355X-native Causal-RoPE + chunk attention (hand-written HIP behind a C ABI).

``binding`` holds the ctypes marshalling for the calls declared in include/crope.h;
``workloads`` the seeded synthetic inputs; ``build`` compiles libcrope.so with hipcc.
Importing the package does not load the library; the first call does, and fails loudly
if it cannot.
"""
from .binding import (  # noqa: F401
    CropeError, TableDesc, chunk_attention, chunk_attention_choose_plan, chunk_attention_limited,
    chunk_attention_planned, chunk_attention_planned_workspace_bytes, chunk_attention_static,
    chunk_attention_static_capacity, chunk_attention_workspace_bytes, crope_build_table,
    CROPE_SCALE_FOLDED, crope_folded_q_scale, crope_last_error, crope_qk_norm_rotate_append, crope_qk_norm_rotate_append_qscaled, crope_qkv_project_norm_rotate_append,
    crope_qkv_project_workspace_bytes, crope_table_bytes, crope_version, library_path,
)
