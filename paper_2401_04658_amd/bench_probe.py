"""ctypes wrapper of libla2_bench.so: the benchmark's measurement kernels (a streaming-only kernel and a
register-only MFMA loop).  Not part of the method and not part of the C ABI of include/la2.h."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libla2_bench.so")
_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError("%s not found (python -m paper_2401_04658_amd.build)" % _LIB_PATH)
        lib = ctypes.CDLL(_LIB_PATH)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
        lib.la2_bench_stream_probe.argtypes = [i32, i32, i32, vp, vp, sz, vp]
        lib.la2_bench_stream_probe.restype = ctypes.c_int
        lib.la2_bench_mfma_peak.argtypes = [i32, i32, vp, vp]
        lib.la2_bench_mfma_peak.restype = ctypes.c_int
        _lib = lib
    return _lib


def _stream(t):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def stream_probe(reads, writes, src, dst, bytes_per_stream, nt_stores=False):
    """One launch of a kernel that only streams `reads` streams out of src and `writes` streams into dst (uint8
    tensors on the GPU, large enough for that many streams of bytes_per_stream)."""
    lib = load()
    if not (src.is_cuda and dst.is_cuda):
        raise ValueError("stream_probe: buffers must live on the GPU")
    if src.numel() * src.element_size() < reads * bytes_per_stream or \
            dst.numel() * dst.element_size() < max(writes * bytes_per_stream, 16):
        raise ValueError("stream_probe: buffer smaller than the streams asked for")
    with torch.cuda.device(src.device):
        rc = lib.la2_bench_stream_probe(reads, writes, 1 if nt_stores else 0, src.data_ptr(), dst.data_ptr(),
                                        bytes_per_stream, _stream(src))
    if rc != 0:
        raise RuntimeError("la2_bench_stream_probe: status %d" % rc)


def mfma_peak(workgroups, iters, sink):
    """One launch of the register-only v_mfma_f32_32x32x16_bf16 loop; returns the FLOPs of the launch."""
    lib = load()
    with torch.cuda.device(sink.device):
        rc = lib.la2_bench_mfma_peak(workgroups, iters, sink.data_ptr(), _stream(sink))
    if rc != 0:
        raise RuntimeError("la2_bench_mfma_peak: status %d" % rc)
    return workgroups * 4 * iters * 16 * 32768
