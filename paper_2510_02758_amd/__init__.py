"""MI355X-native paged KV-cache swap (preempt / write-through / resume).

`paper_2510_02758_amd.kvswap` is the ctypes binding of the C-ABI library built
from `csrc/`; `paper_2510_02758_amd.workloads` holds the seeded synthetic
inputs.  Nothing is imported eagerly: the binding loads the HIP shared object
and fails loudly when it has not been built.
"""
__all__ = ["kvswap", "workloads"]
