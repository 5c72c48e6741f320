"""fp64 CPU oracle for the GSPN scan: test infrastructure, never on the product path."""
from .gspn_oracle import (  # noqa: F401
    scan_fwd, scan_bwd, scan_canonical, scan_canonical_bwd, dense_fwd,
    eq3_block_matrix, one_step_matrix_image, tridiagonal,
    DIR_TB, DIR_BT, DIR_LR, DIR_RL,
)
