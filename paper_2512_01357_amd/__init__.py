"""MI355X-native Load path of the Reuse Store (tensor-level reuse out of a
unified GPU memory pool): a C-ABI HIP library plus this thin Python binding.

``tangram``  ctypes binding, same names as include/tangram.h
``loader``   device slab + streams around the binding (PyTorch as plumbing)
``runner``   replays a synthetic workload
``synth``    seeded synthetic model-shaped inputs
``build``    hipcc build of libtangram.so
"""
__all__ = ["tangram", "loader", "runner", "synth", "build"]
