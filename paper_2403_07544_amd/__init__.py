"""MI355X (gfx950) library for the routed encoder-decoder training step of modular translation
models: hand-written HIP kernels behind a C ABI (include/mammoth_hip.h) plus this thin binding."""
from .binding import (Context, MMError, context_from_setup, load_library, EXPORTS, LIB_PATH,  # noqa: F401
                      KERNEL_CLASSES, MM_OK, MM_EINVAL, MM_ENOMEM, MM_ESTATE, MM_ERANGE, MM_ENONFINITE, MM_EHIP)
