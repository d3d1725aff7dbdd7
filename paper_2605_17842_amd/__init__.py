"""MI355X-native SNLP iteration: thin Python binding over the C ABI of libsnlp_hip.so."""
from .binding import (IDN, HCN, F32, BF16, INIT_H0, INIT_FWD, SnlpError, Snlp, correction_scan_static, load_library, library_path, STAGE_NAMES, N_STAGES)  # noqa: F401
