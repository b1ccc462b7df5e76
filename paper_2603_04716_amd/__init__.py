"""MI355X-native layer-forward library (prefill + decode over a KV cache) and the P/D allocation
model, behind the C ABI declared in include/pd.h."""
from .binding import *  # noqa: F401,F403
from .binding import lib, PdError, EXPORTS  # noqa: F401
