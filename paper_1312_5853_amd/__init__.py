"""MI355X-native convolution hot path (forward, backward-data, backward-filter)
for the ConvNet trained in "Multi-GPU Training of ConvNets" (arXiv 1312.5853).

``paper_1312_5853_amd.binding`` is the thin ctypes layer over the C-ABI library
built from ``csrc/``; ``paper_1312_5853_amd.synth`` draws seeded synthetic
inputs at the network's layer shapes.
"""
