"""MI355X-native block-sparse attention on a lat-lon grid (gfx950 HIP kernels
behind a C ABI).  The Python layer only marshals arguments; see binding.py."""
from .binding import (BsaError, Params, library_path, load_library,  # noqa: F401
                      mosaic_bsa_bwd, mosaic_bsa_bwd_three_branch,
                      mosaic_bsa_check_selection, mosaic_bsa_fwd,
                      mosaic_bsa_fwd_three_branch,
                      mosaic_bsa_probe_mfma, mosaic_bsa_select,
                      mosaic_bsa_select_static, mosaic_bsa_strerror,
                      mosaic_bsa_three_branch_bwd_workspace_bytes,
                      mosaic_bsa_three_branch_workspace_bytes,
                      mosaic_bsa_workspace_bytes)
