"""MI355X-native SAMA meta-gradient step: thin ctypes binding over libsama.so (see include/sama.h)."""
from .binding import (Sama, SamaConfig, SamaError, load_library, lib_path, MODEL_MLP, MODEL_ENCODER, DTYPE_FP32,
                      DTYPE_BF16, OPT_SGD, OPT_ADAM, ADAPT_OPTIMIZER, ADAPT_NONE, STATE)
