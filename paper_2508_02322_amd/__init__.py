"""MI355X-native CAMERA micro-expert scoring path: HIP kernels behind a C ABI
(csrc/, include/camera.h) and a thin ctypes binding (binding.py)."""
