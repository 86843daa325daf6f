"""MI355X-native MGRIT solve over a GRU hidden-state sequence (HIP kernels behind a C ABI)."""
from .binding import (  # noqa: F401
    MgritGruCfg,
    MgritGruError,
    gru_serial_scan,
    gru_serial_scan_backward,
    gru_serial_scan_backward_steps,
    lib,
    lib_path,
    mgrit_gru_backward,
    mgrit_gru_backward_steps,
    mgrit_gru_forward,
    mgrit_gru_profile_enable,
    mgrit_gru_profile_read,
    mgrit_gru_profile_read_shape,
    mgrit_gru_strerror,
    mgrit_gru_workspace_bytes,
)
