"""The GPU tests' helpers live in sfi_check.py at the repository root (bench.py and the smoke check use them too)."""
from sfi_check import *  # noqa: F401,F403
from sfi_check import OUT_TOL, TIE_BAND, Runner, check_out, check_out_bf16, check_selection, i32_dev, make_paged, row_rel_err, to_dev  # noqa: F401
