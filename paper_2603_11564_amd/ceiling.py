"""ctypes binding for libdapq_ceiling.so: the stream and instruction-issue probes that `bench.py --ceilings` reports.
Measurement support only; nothing of the eviction path uses it.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libdapq_ceiling.so")
_lib = None

EXPORTS = ("dapq_ceiling_last_error", "dapq_ceiling_stream", "dapq_ceiling_slice", "dapq_ceiling_num_mixes",
           "dapq_ceiling_slice_mix")


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2603_11564_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    lib.dapq_ceiling_last_error.restype = C.c_char_p
    lib.dapq_ceiling_stream.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.POINTER(C.c_double)]
    lib.dapq_ceiling_slice.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double)]
    lib.dapq_ceiling_slice_mix.restype = C.c_char_p
    lib.dapq_ceiling_slice_mix.argtypes = [C.c_int, C.POINTER(C.c_int)]
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise RuntimeError("libdapq_ceiling: " + load_library().dapq_ceiling_last_error().decode())


def stream(tensor, path, param, waves_per_simd=0, warm=3, reps=20):
    """Reads the tensor's bytes (a multiple of 1 MiB).  path 0: plain loads from `param` workgroups of 256 lanes;
    path 1: the score kernels' LDS ring with `param` slots at `waves_per_simd` waves per SIMD.
    Returns {ms, ghz, gbs}."""
    out = (C.c_double * 5)()
    nbytes = tensor.numel() * tensor.element_size()
    _check(load_library().dapq_ceiling_stream(tensor.data_ptr(), nbytes, path, param, waves_per_simd, warm, reps, out))
    return {"ms": out[0], "ghz": out[1], "gbs": out[3]}


def slice_mixes():
    lib = load_library()
    res = []
    for i in range(lib.dapq_ceiling_num_mixes()):
        counts = (C.c_int * 5)()
        name = lib.dapq_ceiling_slice_mix(i, counts).decode()
        res.append({"index": i, "name": name, "mfma": counts[0], "exp": counts[1], "fma": counts[2], "add": counts[3],
                    "scalar": counts[4]})
    return res


def slice_probe(mix, waves_per_simd, iters=400, warm=3, reps=300):
    """The score passes' slice without memory traffic.  Returns {ms, ghz, ns_per_slice, cycles_per_slice}."""
    out = (C.c_double * 5)()
    _check(load_library().dapq_ceiling_slice(mix, waves_per_simd, iters, warm, reps, out))
    return {"ms": out[0], "ghz": out[1], "ns_per_slice": out[3], "cycles_per_slice": out[4]}
