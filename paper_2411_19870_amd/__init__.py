"""MI355X-native DeMo per-step compression path (encode / decode / step).

`binding` is the thin ctypes layer over libdemo.so (HIP kernels + C ABI);
`synth` holds the seeded synthetic-input generators; `build` compiles the library.
Nothing is loaded at import time; the first call into `binding` loads the shared
library and raises if it has not been built.
"""
