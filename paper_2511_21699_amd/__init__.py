"""MI355X-native tree verification for Cacheback speculative decoding (arXiv 2511.21699).

The product is the C-ABI library built from ``csrc/`` (see ``include/cacheback.h``);
``binding`` is its thin ctypes wrapper.  ``workloads`` and ``drafter`` generate synthetic inputs
on the host.  Nothing is loaded at import time: ``binding.load()`` fails loudly when the HIP
library has not been built.
"""
__all__ = ["binding", "workloads", "drafter", "build"]
