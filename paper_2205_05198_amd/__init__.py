"""MI355X-native selective-activation-recomputation hot path (arXiv 2205.05198, Sections 4.1, 4.2.2, 5).

The package is a thin ctypes binding over ``libsar.so`` (hand-written HIP kernels for gfx950 behind the C ABI
of ``include/sar.h``).  Importing the package does not load the library; the first call does, and fails
loudly if the library has not been built (``python -c "import __graft_entry__ as g; g.build()"``).
"""
from .binding import (  # noqa: F401
    AttnDesc, RowsDesc, SarError, attn_core_bwd_recompute, attn_core_bwd_recompute_dkdv, attn_core_bwd_recompute_dq,
    attn_core_bwd_stored, attn_core_bwd_workspace, attn_core_bwd_workspace_min, attn_core_bwd_noalloc_max_bytes, attn_core_bwd_recompute_noalloc, attn_core_bwd_recompute_stages, sar_test_force_variants,
    attn_core_fwd, attn_core_fwd_stored, attn_core_philox_count, attn_core_saved_bytes,
    attn_core_small_buffer_bytes, bias_dropout_add, bias_dropout_add_bwd, bias_dropout_add_bwd_workspace,
    bias_dropout_add_ln_fwd, bias_gelu_bwd, bias_gelu_bwd_workspace, bias_gelu_fwd, build_library, library_path, ln_bwd, ln_bwd_workspace,
    ln_fwd, load_library, sar_bench_copy, sar_bench_issue, sar_bench_issue_names, sar_bench_mfma, sar_last_error,
)
