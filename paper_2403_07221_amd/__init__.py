"""MI355X-native LookupFFN inference forward pass (hash + table gather).

The compute lives in the C-ABI library built from ``csrc/`` (hand-written HIP
for gfx950); this package is only the argument-marshalling binding around it,
the seeded synthetic-input recipes and the analytic cost model.  Nothing is
loaded at import time: the binding loads the shared library on first use and
raises if it has not been built.
"""
__version__ = "0.1.0"
