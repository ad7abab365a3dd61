"""ctypes binding of ``include/coopt_probe.h`` (libcoopt_probe.so): the streaming-read probe the
benchmark quotes the decode kernels' bandwidth beside.  A measurement aid, no part of the method."""
from __future__ import annotations

import ctypes
import os

from .binding import CooptError, _dev, _nbytes, _stream

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcoopt_probe.so")
_lib = None

EXPORTS = ["coopt_stream_read_probe"]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise CooptError(f"{_LIB_PATH} is not built; run `python -m paper_2602_09323_amd.build`")
        lib = ctypes.CDLL(_LIB_PATH)
        vp = ctypes.c_void_p
        lib.coopt_stream_read_probe.argtypes = [vp, ctypes.c_size_t, ctypes.c_int32, vp, vp]
        lib.coopt_stream_read_probe.restype = ctypes.c_int
        _lib = lib
    return _lib


def stream_read_probe(buf, workgroups: int, sink, stream=None) -> None:
    """One streaming read of the whole tensor ``buf``."""
    status = load_library().coopt_stream_read_probe(
        _dev(buf, "stream_read_probe: buf"), _nbytes(buf), int(workgroups),
        _dev(sink, "stream_read_probe: sink", min_bytes=4), _stream(stream))
    if status != 0:
        raise CooptError(f"coopt_stream_read_probe: status {status}")
