"""FP64 CPU oracle for attention forward.  TEST INFRASTRUCTURE ONLY.

Nothing on the product path imports this package; only tests, the smoke check
and the benchmark's CPU-baseline leg do.  It shares no code with the HIP
library.
"""
from .ref import (Oracle, attn_ref, attn_ref_probs, attn_ref_rows, build,  # noqa: F401
                  compile_c, default, threads, SRC, SO)
