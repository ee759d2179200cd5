"""MI355X-native speculative draft-then-verify denoising round of TS-DP (HIP kernels behind a C ABI)."""
from .binding import EXPORTS, LIB_PATH, Tsdp, TsdpConfig, TsdpError, load_library  # noqa: F401
