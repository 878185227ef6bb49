"""MI355X-native draft-then-verify hot path of multi-layer-draft-head speculative decoding.

The work is done by `libkoala.so` (hand-written HIP for gfx950, C ABI in
`include/koala.h`); this package is the thin Python binding over it.  PyTorch is
used only to own device memory and streams.
"""
from .binding import (KoalaContext, KoalaError, load_library, library_path, measure_stream_read,  # noqa: F401
                      weights_to_f16,
                      KOALA_FP32, KOALA_BF16, KOALA_DRAFT_EAGLE, KOALA_DRAFT_MEDUSA, EXPORTS,
                      Discriminator, MedusaHeadTrainer)
from .packing import (pack_target_weights, pack_eagle_weights, pack_medusa_weights, alloc_kv,  # noqa: F401
                      fragment_major, device_matrix)
