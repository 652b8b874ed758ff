"""ctypes binding of libasd_probe.so (include/asd_probe.h): a measurement probe for the benchmark
harness, separate from the sampling library."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libasd_probe.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libasd_probe.so is not built: run `python -m paper_2505_03983_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.asd_probe_mfma_ceiling.restype = C.c_int32
        L.asd_probe_mfma_ceiling.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.asd_probe_last_error.restype = C.c_char_p
        L.asd_probe_last_error.argtypes = []
        _lib = L
    return _lib


def asd_probe_mfma_ceiling(dtype, random_data=True, ms_target=200):
    """TFLOP/s a register-only MFMA loop sustains on the current device.  dtype: 0 / False fp32, 1 / True bf16, 2 fp16."""
    t = C.c_double(0.0)
    rc = lib().asd_probe_mfma_ceiling(int(dtype), int(bool(random_data)), int(ms_target), C.addressof(t))
    if rc != 0:
        raise RuntimeError("asd_probe_mfma_ceiling failed (%d): %s" % (rc, lib().asd_probe_last_error().decode()))
    return t.value
