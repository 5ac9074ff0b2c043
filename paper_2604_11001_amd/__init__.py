"""MI355X-native Monte-Carlo engine for flow-controlled LLM-inference scheduling.

The product is ``libfcs.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/fcs.h``); this package is its thin ctypes binding.
"""
from .binding import (Engine, FcsError, POLICY_FLOW, POLICY_GREEDY, counter_names, lib,  # noqa: F401
                      protect_limit, stability_bound, strerror)
