"""kvc: head-variable paged decode + block eviction for MI355X (gfx950).

The compute lives in the HIP library built from csrc/ and reached through
`paper_2410_00161_amd.binding` (ctypes, argument marshalling only).  Importing
this package loads nothing; the library is loaded on first use and a missing
library is an error, never a fallback.
"""

__all__ = ["binding", "session", "workloads", "build"]
