"""MI355X-native window-scoring pass of PPOW drafter optimisation (HIP, gfx950).

The product is libppow.so (C ABI declared in include/ppow.h); this package is
the thin Python binding over it.
"""
from .binding import (PPOW_BF16, PPOW_F32, PPOW_FLAG_EXPECTED_ACCEPT,  # noqa: F401
                      PPOW_FLAG_POLICY_TERMS, PPOW_STATIC_MAX_ROWS,
                      PPOW_VERIFY_GREEDY, PPOW_VERIFY_REJECTION, PpowError, ScoreBuffers,
                      SelectBuffers, SequenceBuffers, last_row_kernel, lib,
                      ppow_adaw_sequence, ppow_score_windows, ppow_score_windows_static,
                      ppow_select_windows)
