"""MI355X-native stage kernel of Jupiter's intra-sequence pipeline parallelism.

``binding`` is the thin ctypes layer over the C-ABI library declared in
``include/jupiter_stage.h``; ``synth_inputs`` draws the seeded synthetic tensors.
"""
