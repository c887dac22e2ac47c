"""MI355X-native DRACO encode/decode path (arXiv 1803.09877).

``paper_1803_09877_amd.binding`` loads the HIP library and exposes its C-ABI
entry points; ``paper_1803_09877_amd.synth`` makes seeded synthetic inputs.
Nothing is imported eagerly so that the input generators can be used on a
machine without the built library.
"""
