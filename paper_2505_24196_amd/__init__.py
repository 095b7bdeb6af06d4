"""MI355X-native hot path of CLaSp (in-context layer skip for self-speculative decoding): HIP kernels behind the C
ABI of include/clasp.h, a ctypes binding with the same names, and the host-side draft/verify/optimise loop."""
from .binding import CLASP_BF16, CLASP_F32, ClaspError, Engine, clasp_pack_gate_up, clasp_pack_matrix, lib  # noqa: F401
from .decode import (clasp_generate, clasp_sample_generate, greedy_generate, prefill,  # noqa: F401
                     skip_set_jaccard)
