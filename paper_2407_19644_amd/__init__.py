"""MI355X-native unaligned block-pruned (UBP) sparse x dense product.

Thin ctypes binding over the C ABI declared in include/ubp.h.  Everything is computed by
the native library (host packer + HIP kernels); this package only marshals arguments.
"""
from .binding import (UBPError, Packed, Plan, load_library, library_path, select_reference,  # noqa: F401
                      target_block_count, pack, spmm, spmm_prepare, launch_floor, status_string, layout_slot, DTYPES,
                      EXPORTS, HOST_ONLY, block_scores, select_greedy, select_bed, select_optimal,
                      selection_to_blocks, select_blocks, selection_efficacy, SELECT_METHODS, spmm_fused, Epilogue,
                      ACTIVATIONS)
