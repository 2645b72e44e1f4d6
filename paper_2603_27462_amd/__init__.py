"""MI355X-native RSR (Redundant Segment Reduction) low-bit matvec.

The product is the C-ABI library ``librsr.so`` (``include/rsr.h``); this
package only marshals arguments to it.  There is no CPU fallback: if the
library cannot be loaded every call raises.
"""
from .binding import (  # noqa: F401
    RSR_BINARY, RSR_TERNARY_2PASS, RSR_TERNARY_FUSED, RSR_DENSE_TERNARY_P2,
    RSR_F32, RSR_BF16, RsrError, Handle, load_library, exported_symbols,
    rsr_preprocess, rsr_preprocess_transposed, rsr_preprocess_into, rsr_matvec, rsr_matvec_ex, rsr_destroy,
    rsr_serialize, rsr_deserialize, rsr_last_error,
    rsr_error_string, rsr_get_perm, rsr_get_offsets, rsr_get_packed,
    rsr_num_blocks, rsr_block_height, rsr_num_patterns, rsr_num_passes, rsr_algorithmic_bytes,
    rsr_kernel_name, rsr_launch_shape, rsr_probe_empty, rsr_probe_read,
    rsr_preprocess_stacked, rsr_matvec_stacked,
)
