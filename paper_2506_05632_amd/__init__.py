"""List-level Gumbel-max coupling (GLS) on MI355X: Python binding of the HIP library."""
from .binding import (FLAG_DRAFT_ONLY, FLAG_DRY_RUN, FLAG_EXACT_SCAN, FLAG_MIN_FIRST, FLAG_SHARED_RACE, FLAG_STRONG, LlcError, llc_couple, llc_couple_static, llc_compress_select, llc_couple_is, llc_couple_topm,  # noqa: F401
                      llc_couple_workspace_size, llc_lml_bound, llc_lml_workspace_size, llc_status_string, llc_verify,
                      llc_verify_workspace_size, llc_version, load,
                      new_stats, new_workspace)
