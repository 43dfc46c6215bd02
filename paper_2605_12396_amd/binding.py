"""Thin ctypes binding of libnz.so (include/nz.h).  Argument marshalling only.

PyTorch is used for device memory and streams: tensors are handed over as raw
device pointers, the current HIP stream as a void*.  There is no CPU fallback:
if the library has not been built (python -m paper_2605_12396_amd.build or
__graft_entry__.build()) loading raises.
"""
import ctypes as C
import os

import torch

OK, ERR_INVALID, ERR_CAPACITY, ERR_CORRUPT, ERR_MISMATCH, ERR_HIP = range(6)
RAW, FIXEDLEN, HUFFMAN = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnz.so")


class Opts(C.Structure):
    _fields_ = [("chunk_elems", C.c_uint32), ("seg_syms", C.c_uint32), ("alphabet", C.c_uint32),
                ("force_codec", C.c_int32), ("min_gain_permil", C.c_uint32), ("huff_min_bytes", C.c_uint32),
                ("predictor", C.c_uint32), ("reserved", C.c_uint32)]


def make_opts(chunk_elems=0, seg_syms=0, alphabet=0, force_codec=-1, min_gain_permil=0, huff_min_bytes=0, predictor=0,
              reserved=0):
    return Opts(chunk_elems, seg_syms, alphabet, force_codec, min_gain_permil, huff_min_bytes, predictor, reserved)


class ReaOpts(C.Structure):
    _fields_ = [("sample_bytes", C.c_uint32), ("small_batch_bytes", C.c_uint32), ("link_ps_per_byte", C.c_uint32),
                ("fixed_alpha_ns", C.c_uint32), ("fixed_ps_per_byte", C.c_uint32), ("huff_alpha_ns", C.c_uint32),
                ("huff_ps_per_byte", C.c_uint32), ("reserved", C.c_uint32)]


RESULT_BYTES = 32   # sizeof(nz_result)
REA_RESULT_BYTES = 40   # sizeof(nz_rea_result)
_lib = None


def lib():
    """Load libnz.so (once).  Raises if it is missing: the product path has no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libnz.so is not built: run __graft_entry__.build() (hipcc --offload-arch=gfx950)")
        L = C.CDLL(LIB_PATH)
        vp, sz, f32, po = C.c_void_p, C.c_size_t, C.c_float, C.POINTER(Opts)
        L.nz_version.restype = C.c_uint32
        L.nz_compress_bound.argtypes = [sz, po]
        L.nz_compress_bound.restype = sz
        L.nz_workspace_bytes.argtypes = [sz, po]
        L.nz_workspace_bytes.restype = sz
        L.nz_reduce_workspace_bytes.argtypes = [sz, po]
        L.nz_reduce_workspace_bytes.restype = sz
        L.nz_compress.argtypes = [vp, sz, f32, vp, sz, vp, po, vp, sz, vp]
        L.nz_compress.restype = C.c_int
        L.nz_static_scratch_bytes.restype = sz
        L.nz_compress_static.argtypes = [vp, sz, f32, vp, sz, vp, po, vp]
        L.nz_compress_static.restype = C.c_int
        L.nz_qsgd_step.argtypes = [vp, sz, C.c_uint32, vp, vp, sz, vp]
        L.nz_qsgd_step.restype = C.c_int
        L.nz_compress_sr.argtypes = [vp, sz, f32, C.c_uint32, vp, sz, vp, po, vp, sz, vp]
        L.nz_compress_sr.restype = C.c_int
        L.nz_decompress_step.argtypes = [vp, sz, vp, sz, f32, vp, po, vp, sz, vp]
        L.nz_decompress_step.restype = C.c_int
        L.nz_reduce_frames_step.argtypes = [vp, sz, vp, sz, vp, sz, sz, f32, vp, po, vp, sz, vp]
        L.nz_reduce_frames_step.restype = C.c_int
        L.nz_context_bytes.restype = sz
        L.nz_context_build.argtypes = [vp, sz, f32, po, vp, vp, sz, vp]
        L.nz_context_build.restype = C.c_int
        L.nz_rea_workspace_bytes.argtypes = [sz, po]
        L.nz_rea_workspace_bytes.restype = sz
        L.nz_compress_rea.argtypes = [vp, sz, f32, vp, vp, sz, vp, po, C.POINTER(ReaOpts), vp, sz, vp]
        L.nz_compress_rea.restype = C.c_int
        L.nz_reduce_rea_workspace_bytes.argtypes = [sz, po]
        L.nz_reduce_rea_workspace_bytes.restype = sz
        L.nz_reduce_local_rea.argtypes = [vp, sz, vp, sz, f32, vp, vp, sz, vp, po, C.POINTER(ReaOpts), vp, sz, vp]
        L.nz_reduce_local_rea.restype = C.c_int
        L.nz_decompress.argtypes = [vp, sz, vp, sz, f32, vp, po, vp, sz, vp]
        L.nz_decompress.restype = C.c_int
        L.nz_reduce_frames.argtypes = [vp, sz, vp, sz, vp, sz, sz, f32, vp, po, vp, sz, vp]
        L.nz_reduce_frames.restype = C.c_int
        L.nz_reduce_k.argtypes = [vp, vp, C.c_uint32, vp, sz, sz, f32, vp, po, vp, sz, vp]
        L.nz_reduce_k.restype = C.c_int
        L.nz_reduce_k_step.argtypes = [vp, vp, C.c_uint32, vp, sz, sz, f32, vp, po, vp, sz, vp]
        L.nz_reduce_k_step.restype = C.c_int
        L.nz_reduce_local.argtypes = [vp, sz, vp, vp, sz, sz, f32, vp, po, vp, sz, vp]
        L.nz_reduce_local_sr.argtypes = [vp, sz, vp, vp, sz, sz, f32, C.c_uint32, vp, po, vp, sz, vp]
        L.nz_reduce_local_sr.restype = C.c_int
        L.nz_reduce_local.restype = C.c_int
        L.nz_trace_events.argtypes = [C.POINTER(C.c_void_p), sz]
        L.nz_trace_events.restype = None
        L.nz_trace_recorded.restype = sz
        _lib = L
    return _lib


def _po(opts):
    return C.byref(opts) if opts is not None else None


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def nz_compress_bound(n, opts=None):
    return int(lib().nz_compress_bound(n, _po(opts)))


def nz_workspace_bytes(n, opts=None):
    return int(lib().nz_workspace_bytes(n, _po(opts)))


def nz_reduce_workspace_bytes(n, opts=None):
    return int(lib().nz_reduce_workspace_bytes(n, _po(opts)))


def nz_compress(d_in, n, eb, d_out, out_cap, d_res, opts, d_ws, ws_bytes, stream=None):
    """d_in: float32 cuda tensor; d_out, d_ws: uint8 cuda tensors; d_res: uint8 cuda tensor of RESULT_BYTES."""
    return int(lib().nz_compress(d_in.data_ptr(), n, C.c_float(eb), d_out.data_ptr(), out_cap, d_res.data_ptr(),
                                 _po(opts), d_ws.data_ptr(), ws_bytes, _stream(stream)))


def nz_static_scratch_bytes():
    return int(lib().nz_static_scratch_bytes())


def nz_compress_static(d_in, n, eb, d_out, out_cap, d_res, opts, stream=None):
    """nz_compress with the library's resident scratch array as workspace (allocates nothing)."""
    return int(lib().nz_compress_static(d_in.data_ptr(), n, C.c_float(eb), d_out.data_ptr(), out_cap, d_res.data_ptr(),
                                        _po(opts), _stream(stream)))


def nz_qsgd_step(d_in, n, levels, d_step, d_ws, ws_bytes, stream=None):
    return int(lib().nz_qsgd_step(d_in.data_ptr(), n, levels, d_step.data_ptr(), d_ws.data_ptr(), ws_bytes, _stream(stream)))


def nz_compress_sr(d_in, n, step, seed, d_out, out_cap, d_res, opts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_compress_sr(d_in.data_ptr(), n, C.c_float(step), seed, d_out.data_ptr(), out_cap, d_res.data_ptr(),
                                    _po(opts), d_ws.data_ptr(), ws_bytes, _stream(stream)))


def nz_decompress_step(d_stream, stream_bytes, d_out, n, step, d_res, opts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_decompress_step(d_stream.data_ptr(), stream_bytes, d_out.data_ptr(), n, C.c_float(step),
                                        d_res.data_ptr(), _po(opts), d_ws.data_ptr(), ws_bytes, _stream(stream)))


def nz_reduce_frames_step(d_a, a_bytes, d_b, b_bytes, d_out, out_cap, n, step, d_res, opts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_reduce_frames_step(d_a.data_ptr(), a_bytes, d_b.data_ptr(), b_bytes, d_out.data_ptr(), out_cap, n,
                                           C.c_float(step), d_res.data_ptr(), _po(opts), d_ws.data_ptr(), ws_bytes,
                                           _stream(stream)))


def nz_context_bytes():
    return int(lib().nz_context_bytes())


def nz_context_build(d_sample, n_sample, eb, opts, d_ctx, d_ws, ws_bytes, stream=None):
    return int(lib().nz_context_build(d_sample.data_ptr(), n_sample, C.c_float(eb), _po(opts), d_ctx.data_ptr(),
                                      d_ws.data_ptr(), ws_bytes, _stream(stream)))


def nz_rea_workspace_bytes(n, opts=None):
    return int(lib().nz_rea_workspace_bytes(n, _po(opts)))


def nz_compress_rea(d_in, n, eb, d_ctx, d_out, out_cap, d_res, opts, ropts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_compress_rea(d_in.data_ptr(), n, C.c_float(eb), d_ctx.data_ptr() if d_ctx is not None else None,
                                     d_out.data_ptr(), out_cap, d_res.data_ptr(), _po(opts),
                                     C.byref(ropts) if ropts is not None else None, d_ws.data_ptr(), ws_bytes,
                                     _stream(stream)))


def nz_reduce_rea_workspace_bytes(n, opts=None):
    return int(lib().nz_reduce_rea_workspace_bytes(n, _po(opts)))


def nz_reduce_local_rea(d_in, in_bytes, d_local, n, eb, d_ctx, d_out, out_cap, d_res, opts, ropts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_reduce_local_rea(d_in.data_ptr(), in_bytes, d_local.data_ptr(), n, C.c_float(eb),
                                         d_ctx.data_ptr() if d_ctx is not None else None, d_out.data_ptr(), out_cap,
                                         d_res.data_ptr(), _po(opts), C.byref(ropts) if ropts is not None else None,
                                         d_ws.data_ptr(), ws_bytes, _stream(stream)))


def read_rea_result(d_res):
    import struct
    raw = bytes(d_res.cpu().numpy().tobytes()[:REA_RESULT_BYTES])
    sp, wb, st, nfr, nraw, nfix, nhuf, nfb = struct.unpack("<QQIIIIII", raw)
    return dict(span_bytes=sp, wire_bytes=wb, status=st, n_frames=nfr, n_raw=nraw, n_fixed=nfix, n_huff=nhuf, n_fallback=nfb)


def nz_decompress(d_stream, stream_bytes, d_out, n, eb, d_res, opts, d_ws=None, ws_bytes=0, stream=None):
    return int(lib().nz_decompress(d_stream.data_ptr(), stream_bytes, d_out.data_ptr(), n, C.c_float(eb),
                                   d_res.data_ptr(), _po(opts), d_ws.data_ptr() if d_ws is not None else None,
                                   ws_bytes, _stream(stream)))


def nz_reduce_frames(d_a, a_bytes, d_b, b_bytes, d_out, out_cap, n, eb, d_res, opts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_reduce_frames(d_a.data_ptr(), a_bytes, d_b.data_ptr(), b_bytes, d_out.data_ptr(), out_cap, n,
                                      C.c_float(eb), d_res.data_ptr(), _po(opts), d_ws.data_ptr(), ws_bytes,
                                      _stream(stream)))


def _reduce_k(fn, d_streams, stream_bytes, d_out, out_cap, n, width, d_res, opts, d_ws, ws_bytes, stream):
    k = len(d_streams)
    ptrs = (C.c_void_p * max(k, 1))(*[t.data_ptr() for t in d_streams])
    sizes = (C.c_size_t * max(k, 1))(*[int(b) for b in stream_bytes])
    return int(fn(ptrs, sizes, k, d_out.data_ptr(), out_cap, n, C.c_float(width), d_res.data_ptr(), _po(opts),
                  d_ws.data_ptr(), ws_bytes, _stream(stream)))


def nz_reduce_k(d_streams, stream_bytes, d_out, out_cap, n, eb, d_res, opts, d_ws, ws_bytes, stream=None):
    """d_streams: sequence of device tensors, stream_bytes: their sizes (host arrays of pointers / sizes are built here)."""
    return _reduce_k(lib().nz_reduce_k, d_streams, stream_bytes, d_out, out_cap, n, eb, d_res, opts, d_ws, ws_bytes, stream)


def nz_reduce_k_step(d_streams, stream_bytes, d_out, out_cap, n, step, d_res, opts, d_ws, ws_bytes, stream=None):
    return _reduce_k(lib().nz_reduce_k_step, d_streams, stream_bytes, d_out, out_cap, n, step, d_res, opts, d_ws, ws_bytes, stream)


def nz_reduce_local(d_in, in_bytes, d_local, d_out, out_cap, n, eb, d_res, opts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_reduce_local(d_in.data_ptr(), in_bytes, d_local.data_ptr(), d_out.data_ptr(), out_cap, n,
                                     C.c_float(eb), d_res.data_ptr(), _po(opts), d_ws.data_ptr(), ws_bytes,
                                     _stream(stream)))


def nz_reduce_local_sr(d_in, in_bytes, d_local, d_out, out_cap, n, step, seed, d_res, opts, d_ws, ws_bytes, stream=None):
    return int(lib().nz_reduce_local_sr(d_in.data_ptr(), in_bytes, d_local.data_ptr(), d_out.data_ptr(), out_cap, n,
                                        C.c_float(step), seed, d_res.data_ptr(), _po(opts), d_ws.data_ptr(), ws_bytes,
                                        _stream(stream)))


def read_result(d_res):
    """Copy the device result record to the host (synchronises) and unpack it."""
    import struct
    raw = bytes(d_res.cpu().numpy().tobytes()[:RESULT_BYTES])
    b, st, nfr, nraw, nfix, nhuf, _ = struct.unpack("<QIIIIII", raw)
    return dict(bytes=b, status=st, n_frames=nfr, n_raw=nraw, n_fixed=nfix, n_huff=nhuf)


class Session:
    """Caller-owned buffers for repeated calls on messages of up to n elements (a convenience for tests and
    the benchmark; the library itself keeps no state)."""

    def __init__(self, n, opts=None, device="cuda:0", reduce=False):
        self.n, self.opts, self.device = n, opts, torch.device(device)
        self.cap = nz_compress_bound(n, opts)
        self.ws_bytes = nz_reduce_workspace_bytes(n, opts) if reduce else nz_workspace_bytes(n, opts)
        if self.cap == 0 or self.ws_bytes == 0:
            raise ValueError("invalid n/opts")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        self.res = torch.zeros(RESULT_BYTES, dtype=torch.uint8, device=self.device)

    def new_stream_buffer(self):
        return torch.empty(self.cap, dtype=torch.uint8, device=self.device)

    def compress(self, x, eb, out=None, cap=None):
        out = out if out is not None else self.new_stream_buffer()
        rc = nz_compress(x, x.numel(), eb, out, self.cap if cap is None else cap, self.res, self.opts, self.ws,
                         self.ws_bytes)
        return rc, out

    def decompress(self, stream, nbytes, n, eb, out=None):
        out = out if out is not None else torch.empty(n, dtype=torch.float32, device=self.device)
        rc = nz_decompress(stream, nbytes, out, n, eb, self.res, self.opts, self.ws, self.ws_bytes)
        return rc, out

    def reduce(self, a, a_bytes, b, b_bytes, n, eb, out=None, cap=None):
        out = out if out is not None else self.new_stream_buffer()
        rc = nz_reduce_frames(a, a_bytes, b, b_bytes, out, self.cap if cap is None else cap, n, eb, self.res,
                              self.opts, self.ws, self.ws_bytes)
        return rc, out

    def reduce_k(self, streams, sizes, n, eb, out=None, cap=None):
        out = out if out is not None else self.new_stream_buffer()
        rc = nz_reduce_k(streams, sizes, out, self.cap if cap is None else cap, n, eb, self.res, self.opts, self.ws,
                         self.ws_bytes)
        return rc, out

    def reduce_local(self, a, a_bytes, x, n, eb, out=None, cap=None):
        out = out if out is not None else self.new_stream_buffer()
        rc = nz_reduce_local(a, a_bytes, x, out, self.cap if cap is None else cap, n, eb, self.res,
                             self.opts, self.ws, self.ws_bytes)
        return rc, out

    def result(self):
        return read_result(self.res)


class KernelTrace:
    """Per-kernel timing of nz_* calls with HIP events recorded by the library on the call's stream."""

    def __init__(self, max_events=8):
        self.events = [torch.cuda.Event(enable_timing=True) for _ in range(max_events)]
        for e in self.events:
            e.record()                      # torch creates the hipEvent_t lazily at the first record
        torch.cuda.synchronize()
        self.handles = (C.c_void_p * max_events)(*[C.c_void_p(e.cuda_event) for e in self.events])

    def __enter__(self):
        lib().nz_trace_events(self.handles, len(self.events))
        return self

    def __exit__(self, *exc):
        lib().nz_trace_events(None, 0)

    def kernel_ms(self):
        """Durations between consecutive recorded events of the last call (synchronises)."""
        k = int(lib().nz_trace_recorded())
        torch.cuda.synchronize()
        return [self.events[i].elapsed_time(self.events[i + 1]) for i in range(k - 1)]
