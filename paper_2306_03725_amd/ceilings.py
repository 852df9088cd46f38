"""ctypes binding of libusl_ceilings (include/usl_ceilings.h): runs the measurement kernels and
returns their figures as a dict.  Used by bench.py; not part of the training path."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libusl_ceilings.so")
SYMBOLS = ["usl_ceilings_count", "usl_ceilings_name", "usl_ceilings_run"]

if not os.path.exists(LIB_PATH):
    raise ImportError("libusl_ceilings.so is not built: run `python -m paper_2306_03725_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)
_lib.usl_ceilings_count.restype = ctypes.c_int
_lib.usl_ceilings_name.argtypes = [ctypes.c_int]
_lib.usl_ceilings_name.restype = ctypes.c_char_p
_lib.usl_ceilings_run.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int]
_lib.usl_ceilings_run.restype = ctypes.c_int


def names():
    return [_lib.usl_ceilings_name(i).decode() for i in range(_lib.usl_ceilings_count())]


def run():
    """{figure name: value} measured on the current HIP device; raises on a HIP error."""
    n = _lib.usl_ceilings_count()
    vals = (ctypes.c_double * n)()
    rc = _lib.usl_ceilings_run(vals, n)
    if rc != 0:
        raise RuntimeError("usl_ceilings_run failed with hipError_t %d" % rc)
    return dict(zip(names(), (float(v) for v in vals)))
