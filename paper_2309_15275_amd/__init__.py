"""MI355X-native LBP-WHT: low-rank backpropagation through a linear layer with Walsh-Hadamard
projections (hand-written HIP kernels behind a C ABI, see include/lbp_wht.h)."""
from .binding import (  # noqa: F401
    LbpError,
    full_bp_backward,
    lbp_wht_backward,
    lbp_wht_backward_preprojected,
    select_bases,
    select_lhe,
    wht_energy,
    wht_project,
    wht_project_pair,
    wht_unproject,
)
