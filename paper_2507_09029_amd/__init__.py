"""MI355X-native masked-MLP hot path of Subnetwork Data Parallelism: thin binding over libsdp_hip.so."""
from .binding import (  # noqa: F401
    SdpError,
    coverage_grad_avg,
    index_masks,
    index_masks_workspace_bytes,
    lib,
    library_path,
    make_masks,
    masked_mlp_bwd,
    masked_mlp_bwd_workspace_bytes,
    masked_mlp_fwd,
    masked_mlp_fwd_workspace_bytes,
    profile_enable,
    profile_filter,
    profile_read,
    profile_reset,
    sample_masks_host,
)
