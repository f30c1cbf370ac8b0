"""MI355X-native speculative-decoding verification (the hot path of DSSD, arXiv 2507.12000).

`synth` builds seeded synthetic inputs; `binding` is the thin ctypes layer over the HIP
library libdssd.so (include/dssd.h).  Importing the package does not load the library;
`binding.load()` does, and raises if it has not been built.
"""
