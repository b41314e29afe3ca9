"""ctypes binding of libcamera_bench.so (include/camera_bench.h): measured machine ceilings for benchmark
reports.  Apart from the product library on purpose; nothing of the method runs here."""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcamera_bench.so")
EXPORTS = ["camera_bench_mfma_bf16", "camera_bench_hbm_read"]


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2508_02322_amd.build`")
    lib = ctypes.CDLL(path)
    d, i, i64 = ctypes.c_double, ctypes.c_int, ctypes.c_int64
    lib.camera_bench_mfma_bf16.argtypes = [i, i, i, ctypes.POINTER(d), ctypes.POINTER(d)]
    lib.camera_bench_hbm_read.argtypes = [i, i64, i, ctypes.POINTER(d)]
    for name in EXPORTS:
        getattr(lib, name).restype = i
    return lib


def mfma_bf16(random_operands: bool, launches: int = 50, device: int = 0):
    """(TFLOP/s, shader MHz) of the register-resident MFMA loop."""
    tf, mhz = ctypes.c_double(), ctypes.c_double()
    rc = load_library().camera_bench_mfma_bf16(device, int(random_operands), int(launches), ctypes.byref(tf), ctypes.byref(mhz))
    if rc != 0:
        raise RuntimeError(f"camera_bench_mfma_bf16: status {rc}")
    return tf.value, mhz.value


def hbm_read(nbytes: int, launches: int = 10, device: int = 0):
    """GB/s of a streaming read of nbytes."""
    gbs = ctypes.c_double()
    rc = load_library().camera_bench_hbm_read(device, int(nbytes), int(launches), ctypes.byref(gbs))
    if rc != 0:
        raise RuntimeError(f"camera_bench_hbm_read: status {rc}")
    return gbs.value
