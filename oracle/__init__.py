"""CPU oracle for the middle-submodel forward (test infrastructure only).

Everything under this package is a slow, plain restatement of what the hot
path computes.  It exists to check the HIP library; it is never a fallback.
Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import it.  It shares no code with the HIP path and imports nothing from it.
"""
from .decoder import OracleMiddle, rmsnorm, rope_rotate_half, prefix_causal_attention, decoder_layer  # noqa: F401
from .page_model import PageModel, PageModelError  # noqa: F401
