"""MI355X-native verification path of Adaptive N-gram Parallel Decoding.

``synth`` (seeded inputs) imports without the HIP library; ``binding`` loads
``libanpd.so`` and raises if it is missing.
"""
