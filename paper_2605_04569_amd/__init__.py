"""MI355X-native In-Context Sparse Attention: thin Python binding over libisa_hip.so."""
from .binding import (  # noqa: F401
    Grid, IsaError, Problem, lib, lib_path,
    isa_attention, isa_attention_backward, isa_attention_simple, isa_attention_static, isa_attend, isa_block_means, isa_coarse_output, isa_coarse_scores, isa_dense_attention,
    isa_get_counts, isa_prologue, isa_prologue_backward, isa_select, isa_untile, isa_last_attention_kernel_ms, isa_set_mfma, isa_time_attention_kernel, isa_strerror, isa_workspace_bytes, isa_workspace_layout, workspace_array, new_workspace,
)
from .autograd import InContextSparseAttention  # noqa: F401,E402
