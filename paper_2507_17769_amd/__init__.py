"""MI355X-native mixed-batch serving step (chunked prefill + decode over a paged KV cache).

`workloads` draws the seeded synthetic inputs; `binding` is the ctypes layer over
the C-ABI library built from `csrc/` (import it explicitly: it loads the HIP
library and raises if the library has not been built).
"""
