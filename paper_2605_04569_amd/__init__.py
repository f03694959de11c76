"""MI355X-native In-Context Sparse Attention: thin Python binding over libisa_hip.so."""
from .binding import (  # noqa: F401
    IsaError, Problem, lib, lib_path,
    isa_attention, isa_attention_simple, isa_attend, isa_block_means, isa_coarse_scores, isa_dense_attention,
    isa_get_counts, isa_select, isa_set_mfma, isa_strerror, isa_workspace_bytes, new_workspace,
)
