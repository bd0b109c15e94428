"""MI355X-native per-GPU pipeline-stage forward (HexGen hot path).  See include/hexgen.h."""
from .binding import (HEXGEN_BF16, HEXGEN_F32, HexgenError, KVCache, Stage, accumulate_f32, lib, stream_copy, stream_read, mfma_probe,  # noqa: F401
                      LIB_PATH, SIGNATURES)
