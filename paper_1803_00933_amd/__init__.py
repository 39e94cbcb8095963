"""MI355X-native replay memory of Ape-X (distributed prioritized experience replay).

``apex`` is the thin binding of the C-ABI library built from ``csrc/``; ``synth`` draws the
seeded synthetic inputs.  Importing the binding needs the built library and fails loudly
without it, so it is imported on first use rather than here.
"""
