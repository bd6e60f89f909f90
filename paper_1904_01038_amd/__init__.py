"""MI355X-native mixed-precision Transformer training step (thin binding over libtfm.so)."""
from .binding import (Tfm, Decoder, TfmError, TfmConfig, lib, lib_path, make_config,        # noqa: F401
                      FP32, FP16, BF16, PROF_CLASSES, lr_inverse_sqrt, lr_cosine_restarts, batch_by_length, shuffle_batches)
from . import ops                                                                   # noqa: F401
