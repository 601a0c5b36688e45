"""MI355X-native tree-verification step for speculative decoding.

``binding`` holds the ctypes front end of libghd.so (the HIP kernels behind the
C ABI in include/ghd.h); ``workloads`` holds the seeded synthetic inputs;
``build`` compiles the library in-tree.  Nothing is imported eagerly so that the
input generators can be used without the GPU library.
"""
