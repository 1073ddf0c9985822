"""Micro-batched convolution for MI355X (gfx950): hand-written HIP kernels behind a
C-ABI library, after the method of arXiv 1804.04806.

``paper_1804_04806_amd.ucd`` is the ctypes binding (argument marshalling only);
``paper_1804_04806_amd.synth`` holds seeded input generators and workload shapes;
``paper_1804_04806_amd.build`` compiles the library with hipcc.
Nothing is imported eagerly so that shape tables can be used without the library.
"""
