"""MI355X-native quantized training operators (QSync's backend hot path).

The compute lives in the HIP library ``libqsync.so`` (see ``csrc/`` and
``include/qsync.h``); this package only marshals arguments for it.
"""
from . import workloads  # noqa: F401
