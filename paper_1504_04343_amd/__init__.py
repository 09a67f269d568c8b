"""MI355X-native lowering-based convolutional layer (Caffe con Troll's hot path).

``binding``  - ctypes binding of the C-ABI library ``libcct.so`` (HIP kernels for gfx950).
``synth``    - seeded synthetic workloads (no arithmetic of the method).
``build``    - compiles ``csrc/`` with hipcc into ``libcct.so``.

Importing ``binding`` fails loudly if the library has not been built; there is
no CPU fallback anywhere in this package.
"""
