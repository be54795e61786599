"""MI355X-native chunked-prefill decoder-layer library (HIP kernels behind a C ABI) and its thin binding."""
from .binding import (  # noqa: F401
    RsError, LayerConfig, Context, KVCache, PackedWeights, load_library, library_path, STATUS,
)
