"""MI355X-native SLICER intermediate-feature codec (arXiv 2511.11608, Sec. 3).

``binding`` wraps the C ABI of libslicer.so (hand-written HIP for gfx950);
``synth`` generates the seeded synthetic workloads; ``build`` compiles the library.
"""
