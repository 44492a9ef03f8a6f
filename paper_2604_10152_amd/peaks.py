"""ctypes binding of libspecmoe_peaks.so: microbenchmarks of the box's measured ceilings
(bf16 matrix instructions from registers, HBM read stream, L2 -> LDS stream).  Used by
`bench.py --mode peaks` only; argument marshalling, no arithmetic."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def load():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libspecmoe_peaks.so")
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path}: build it with `python -m paper_2604_10152_amd.build`")
        lib = ctypes.CDLL(path)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        lib.specmoe_peak_mfma.argtypes = [i, i, i, vp, vp, ctypes.POINTER(ctypes.c_double), vp]
        lib.specmoe_peak_hbm_read.argtypes = [vp, sz, i, vp, vp]
        lib.specmoe_peak_l2_lds.argtypes = [vp, sz, i, i, i, vp]
        lib.specmoe_peak_l2_lds_nt.argtypes = [vp, sz, i, i, vp]
        lib.specmoe_peak_lds_read.argtypes = [i, i, vp, vp, vp]
        _LIB = lib
    return _LIB


def _check(st, where):
    if st != 0:
        raise RuntimeError(f"{where}: status {st}")


def mfma(kind, blocks, iters, out, clocks, stream):
    flops = ctypes.c_double(0.0)
    _check(load().specmoe_peak_mfma(kind, blocks, iters, out.data_ptr(), clocks.data_ptr(),
                                    ctypes.byref(flops), stream.cuda_stream), "specmoe_peak_mfma")
    return flops.value


def hbm_read(buf, blocks, sink, stream):
    _check(load().specmoe_peak_hbm_read(buf.data_ptr(), buf.numel() * buf.element_size(), blocks,
                                        sink.data_ptr(), stream.cuda_stream), "specmoe_peak_hbm_read")
    return buf.numel() * buf.element_size()


def l2_lds(buf, region_bytes, blocks, iters, seg, stream):
    _check(load().specmoe_peak_l2_lds(buf.data_ptr(), region_bytes, blocks, iters, seg,
                                      stream.cuda_stream), "specmoe_peak_l2_lds")
    return blocks * iters * (256 << 10)


def l2_lds_nt(buf, region_bytes, blocks, iters, stream):
    _check(load().specmoe_peak_l2_lds_nt(buf.data_ptr(), region_bytes, blocks, iters,
                                         stream.cuda_stream), "specmoe_peak_l2_lds_nt")
    return blocks * iters * (256 << 10)


def lds_read(pattern, iters, clocks, sink, stream):
    _check(load().specmoe_peak_lds_read(pattern, iters, clocks.data_ptr(), sink.data_ptr(),
                                        stream.cuda_stream), "specmoe_peak_lds_read")
