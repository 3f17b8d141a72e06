"""MI355X-native Locret chunk step: chunked-prefill attention + retaining head + KV eviction.

`synth` (seeded inputs) imports without the HIP library; everything in `binding`
needs the built shared library and raises if it is missing.
"""
