"""MI355X-native hot path behind OrchMLLM's Batch Post-Balancing Dispatcher:
balance -> pack -> varlen attention, hand-written HIP behind a C ABI."""
from .binding import (  # noqa: F401
    Assignment,
    OrchError,
    attn_variant,
    balance,
    balance_padded,
    balance_static,
    balance_static_max_n,
    balance_tolerance,
    comm_volume,
    balance_workspace,
    library_path,
    load_library,
    pack,
    pack_composed,
    pack_composed_workspace,
    pack_workspace,
    varlen_attn_bwd,
    varlen_attn_bwd_workspace,
    varlen_attn_fwd,
    varlen_attn_workspace,
)
