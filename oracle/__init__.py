"""CPU oracle for Interlaced-Mask (IM) attention, the GsiT encoder layer and the model around it.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, fp64 definition the
GPU library is checked against.  Nothing in the product path may import it: only
the test-suite, the smoke check and the CPU-baseline leg of the benchmark do.
It shares no code, tables or helpers with the HIP implementation and imports
nothing from it.

Every function is the textbook definition written out with numpy (matmul as the
only library primitive), following the paper's Sections "All-Modal-In-One
Fusion", "Information Disorder" and Appendix A; there is no blocking, fusion or
reordering.
"""
from .im_attention import (  # noqa: F401
    IM_IFM_FORWARD, IM_IFM_BACKWARD, IM_IEM, IM_DENSE, NAMED_PATTERNS,
    live_mask_from_edges, segment_of_rows, key_invalid, additive_mask,
    project_qkv, forward, backward, mult_blocks_forward, live_pair_count,
)
from .gsit_layer import (  # noqa: F401
    layer_norm, gelu, gelu_grad, layer_norm_backward, gsit_layer_forward, gsit_layer_backward, gsit_encoder_forward,
)
from .gsit_model import gsit_model_forward, last_steps  # noqa: F401
