"""Python binding of libskv (routed GQA attention over a depth-shared KV cache, MI355X).

Argument marshalling only: every function has the name and meaning of the C entry point declared
in include/skv.h and passes device pointers of torch tensors straight through.  There is no
fallback: if the HIP library cannot be loaded the import of `lib()` raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
