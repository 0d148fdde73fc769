"""MI355X-native implementation of the quantised message path of AdaQP (arXiv 2306.01381).

`binding` mirrors the C ABI of include/adaqp.h, `layer` owns device memory for a layer step, `synth` draws
seeded synthetic partitions.  The HIP library is built in-tree by `python -m paper_2306_01381_amd.build`.
"""
__version__ = "0.1.0"
