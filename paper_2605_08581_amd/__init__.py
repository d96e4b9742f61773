"""MI355X-native prefix-cached prefill attention over a paged KV cache.

The compute lives in the HIP library under ``csrc/`` (C ABI declared in
``include/prism.h``); ``binding`` marshals arguments to it and ``workload``
draws seeded synthetic inputs.  Importing the package loads nothing; the
library is loaded on first use and its absence is an error, never a fallback.
"""
__all__ = ["workload", "binding", "sched", "trace", "replay", "queueing"]
