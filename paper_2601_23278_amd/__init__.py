"""MI355X-native FOCUS decode step: hand-written HIP kernels behind a C ABI (include/focus.h)."""
from .binding import *  # noqa: F401,F403  (raises ImportError when libfocus.so is not built)
from .binding import Focus, FocusError, focus_config, focus_step_out, focus_seq_state, make_step_out  # noqa: F401
