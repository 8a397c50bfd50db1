"""MI355X-native batched KV-cache compression stage (FastCache hot path).

`fastcache` is the ctypes binding over the C-ABI library (include/fastcache.h);
`synth` makes seeded synthetic workloads.  Importing the package does not load
the HIP library; the first use of the binding does, and fails loudly if it has
not been built.
"""
