"""MI355X-native batched decode step over a paged KV cache (the serving
instance's iteration that the Chiron local autoscaler sizes).

`inputs` draws seeded synthetic workloads; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/` by `build`.  Nothing is loaded at
import time; the binding raises if the HIP library has not been built.
"""
