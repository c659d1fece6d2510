"""EasyScaleThread (EST) step on one MI355X: thin Python layer over libes.

``binding``  ctypes mirror of include/es.h (argument marshalling only)
``job``      convenience object that owns the torch tensors and streams a job
             needs and forwards to the binding
``build``    compiles csrc/ into libes.so with hipcc for gfx950

All data movement and arithmetic of the step runs in the HIP kernels of
libes.so; there is no CPU or PyTorch fallback.
"""
