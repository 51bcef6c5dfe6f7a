"""MI355X-native AET-SGD hot path: HIP kernels behind a C ABI (include/aet_sgd.h) and a
thin Python binding with the same names."""
from .binding import AetError, AetSgd, load_library  # noqa: F401
