"""CPU oracle for LBP-WHT.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  The GPU library and its Python binding never do, and this package imports
nothing from them.
"""
from .lbp_oracle import (  # noqa: F401
    build,
    sylvester,
    walsh,
    select_bases,
    basis_matrix,
    project,
    unproject,
    lbp_wht_backward,
    full_bp_backward,
    lbp_gx_tokens,
    lbp_gw_entries,
    full_gx_tokens,
    full_gw_entries,
    flop_model,
    wht_energy,
    select_lhe,
    pad_grid,
    project_padded,
    unproject_padded,
    lbp_wht_backward_padded,
    wht_energy_padded,
    lbp_wht_backward_tokens,
    max_threads,
    set_threads,
)
