"""INT8 convolution backward with distribution-adaptive gradient quantization, native to MI355X.

``binding`` wraps the C ABI of ``libdaq.so`` (include/daq.h); ``workloads`` holds the seeded synthetic
layer shapes and inputs; ``build`` compiles the library.
"""
