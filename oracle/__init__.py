"""ctypes face of the CPU oracle (oracle/nz_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  Nothing in the product package imports it, and it
imports nothing from the product package.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OK, ERR_INVALID, ERR_CAPACITY, ERR_CORRUPT, ERR_MISMATCH = 0, 1, 2, 3, 4
RAW, FIXEDLEN, HUFFMAN = 0, 1, 2
HDR_BYTES = 32
STREAM_HDR = 64


class Opts(C.Structure):
    _fields_ = [("chunk_elems", C.c_uint32), ("seg_syms", C.c_uint32), ("alphabet", C.c_uint32),
                ("force_codec", C.c_int32), ("min_gain_permil", C.c_uint32), ("huff_min_bytes", C.c_uint32),
                ("predictor", C.c_uint32), ("reserved", C.c_uint32)]


class Result(C.Structure):
    _fields_ = [("bytes", C.c_uint64), ("status", C.c_uint32), ("n_frames", C.c_uint32),
                ("n_raw", C.c_uint32), ("n_fixed", C.c_uint32), ("n_huff", C.c_uint32),
                ("reserved", C.c_uint32)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_ if k != "reserved"}


class Context(C.Structure):
    _fields_ = [("valid", C.c_uint32), ("K", C.c_uint32), ("len", C.c_uint8 * 1024), ("code", C.c_uint32 * 1024)]


class ReaOpts(C.Structure):
    _fields_ = [("sample_bytes", C.c_uint32), ("small_batch_bytes", C.c_uint32), ("link_ps_per_byte", C.c_uint32),
                ("fixed_alpha_ns", C.c_uint32), ("fixed_ps_per_byte", C.c_uint32), ("huff_alpha_ns", C.c_uint32),
                ("huff_ps_per_byte", C.c_uint32), ("reserved", C.c_uint32)]


class ReaResult(C.Structure):
    _fields_ = [("span_bytes", C.c_uint64), ("wire_bytes", C.c_uint64), ("status", C.c_uint32), ("n_frames", C.c_uint32),
                ("n_raw", C.c_uint32), ("n_fixed", C.c_uint32), ("n_huff", C.c_uint32), ("n_fallback", C.c_uint32)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


class ReaPlan(C.Structure):
    _fields_ = [("n_s", C.c_uint32), ("sample_ok", C.c_uint32), ("w_s", C.c_uint32), ("sample_bits", C.c_uint64),
                ("pred_payload", C.c_uint64 * 3), ("plan", C.c_int)]


def make_opts(chunk_elems=0, seg_syms=0, alphabet=0, force_codec=-1, min_gain_permil=0, huff_min_bytes=0, predictor=0,
              reserved=0):
    return Opts(chunk_elems, seg_syms, alphabet, force_codec, min_gain_permil, huff_min_bytes, predictor, reserved)


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        vp, sz, f32 = C.c_void_p, C.c_size_t, C.c_float
        L.nzo_step_constants.argtypes = [f32, C.POINTER(f32), C.POINTER(f32)]
        L.nzo_quantize.argtypes = [vp, sz, f32, vp, vp]
        L.nzo_dequantize_one.argtypes = [C.c_int32, f32]
        L.nzo_dequantize_one.restype = f32
        L.nzo_zigzag.argtypes = [C.c_int32]
        L.nzo_zigzag.restype = C.c_uint32
        L.nzo_unzigzag.argtypes = [C.c_uint32]
        L.nzo_unzigzag.restype = C.c_int32
        L.nzo_huffman_lengths.argtypes = [vp, C.c_uint32, vp]
        L.nzo_canonical_codes.argtypes = [vp, C.c_uint32, vp]
        L.nzo_canonical_codes.restype = None
        L.nzo_compress_bound.argtypes = [sz, C.POINTER(Opts)]
        L.nzo_compress_bound.restype = sz
        L.nzo_compress.argtypes = [vp, sz, f32, C.POINTER(Opts), vp, sz, C.POINTER(Result)]
        L.nzo_decompress.argtypes = [vp, sz, vp, sz, f32, C.POINTER(Result)]
        L.nzo_decode_codes.argtypes = [vp, sz, sz, f32, vp, vp, vp, C.POINTER(Result)]
        L.nzo_reduce_frames.argtypes = [vp, sz, vp, sz, vp, sz, sz, f32, C.POINTER(Opts), C.POINTER(Result)]
        L.nzo_reduce_local.argtypes = [vp, sz, vp, vp, sz, sz, f32, C.POINTER(Opts), C.POINTER(Result)]
        L.nzo_reduce_k.argtypes = [vp, vp, C.c_uint32, vp, sz, sz, f32, C.POINTER(Opts), C.POINTER(Result)]
        L.nzo_reduce_k_step.argtypes = [vp, vp, C.c_uint32, vp, sz, sz, f32, C.POINTER(Opts), C.POINTER(Result)]
        L.nzo_frame_plan.argtypes = [vp, C.c_uint32, C.c_int, C.POINTER(Opts), vp, vp, vp, vp, vp, vp, vp]
        L.nzo_frame_encode.argtypes = [vp, vp, C.c_uint32, C.c_int, C.POINTER(Opts), C.c_uint32, vp, sz]
        L.nzo_frame_encode.restype = C.c_int64
        L.nzo_sr_draw.argtypes = [C.c_uint32, C.c_uint64]
        L.nzo_sr_draw.restype = C.c_uint32
        L.nzo_sr_quantize.argtypes = [vp, sz, f32, C.c_uint32, C.c_uint64, vp, vp]
        L.nzo_qsgd_step.argtypes = [vp, sz, C.c_uint32, C.POINTER(f32)]
        L.nzo_compress_sr.argtypes = [vp, sz, f32, C.c_uint32, C.POINTER(Opts), vp, sz, C.POINTER(Result)]
        L.nzo_decompress_step.argtypes = [vp, sz, vp, sz, f32, C.POINTER(Result)]
        L.nzo_decode_codes_step.argtypes = [vp, sz, sz, f32, vp, vp, vp, C.POINTER(Result)]
        L.nzo_reduce_frames_step.argtypes = [vp, sz, vp, sz, vp, sz, sz, f32, C.POINTER(Opts), C.POINTER(Result)]
        L.nzo_reduce_local_sr.argtypes = [vp, sz, vp, vp, sz, sz, f32, C.c_uint32, C.POINTER(Opts), C.POINTER(Result)]
        L.nzo_context_build.argtypes = [vp, sz, f32, C.POINTER(Opts), C.POINTER(Context)]
        L.nzo_rea_plan_frame.argtypes = [vp, C.c_uint32, f32, C.POINTER(Opts), C.POINTER(ReaOpts), C.POINTER(Context),
                                         C.POINTER(ReaPlan)]
        L.nzo_compress_rea.argtypes = [vp, sz, f32, C.POINTER(Opts), C.POINTER(ReaOpts), C.POINTER(Context), vp, sz,
                                       C.POINTER(ReaResult), vp]
        L.nzo_reduce_local_rea.argtypes = [vp, sz, vp, sz, f32, C.POINTER(Opts), C.POINTER(ReaOpts), C.POINTER(Context), vp, sz,
                                           C.POINTER(ReaResult), vp]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def step_constants(eb):
    s, r = C.c_float(), C.c_float()
    rc = lib().nzo_step_constants(C.c_float(eb), C.byref(s), C.byref(r))
    if rc:
        raise ValueError("invalid error bound")
    return np.float32(s.value), np.float32(r.value)


def quantize(x, eb):
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.size, np.int32)
    ok = np.empty(x.size, np.uint8)
    rc = lib().nzo_quantize(_ptr(x), x.size, C.c_float(eb), _ptr(q), _ptr(ok))
    if rc:
        raise ValueError("invalid error bound")
    return q, ok.astype(bool)


def dequantize(q, eb):
    step, _ = step_constants(eb)
    return np.array([lib().nzo_dequantize_one(int(v), C.c_float(step)) for v in np.asarray(q).ravel()], np.float32)


def zigzag(q):
    return int(lib().nzo_zigzag(int(q)))


def unzigzag(z):
    return int(lib().nzo_unzigzag(int(z)))


def huffman_lengths(freq):
    f = np.ascontiguousarray(freq, dtype=np.uint32)
    ln = np.zeros(f.size, np.uint8)
    m = lib().nzo_huffman_lengths(_ptr(f), f.size, _ptr(ln))
    if m < 0:
        raise ValueError("alphabet too large")
    return ln


def canonical_codes(lengths):
    ln = np.ascontiguousarray(lengths, dtype=np.uint8)
    code = np.zeros(ln.size, np.uint32)
    lib().nzo_canonical_codes(_ptr(ln), ln.size, _ptr(code))
    return code


def compress_bound(n, opts=None):
    return int(lib().nzo_compress_bound(n, C.byref(opts) if opts is not None else None))


def compress(x, eb, opts=None, cap=None):
    """Returns (stream bytes as np.uint8 array trimmed to its length, Result, rc)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if cap is None:
        cap = compress_bound(x.size, opts)
    out = np.zeros(max(cap, 1), np.uint8)
    res = Result()
    rc = lib().nzo_compress(_ptr(x), x.size, C.c_float(eb), C.byref(opts) if opts is not None else None,
                            _ptr(out), cap, C.byref(res))
    return out[:res.bytes].copy(), res, rc


def decompress(stream, n, eb):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    out = np.zeros(n, np.float32)
    res = Result()
    rc = lib().nzo_decompress(_ptr(s), s.size, _ptr(out), n, C.c_float(eb), C.byref(res))
    return out, res, rc


def decode_codes(stream, n, eb):
    """Returns (q int32[n], rawbits uint32[n], frame_kind uint8[n_frames], Result, rc)."""
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    q = np.zeros(n, np.int32)
    rb = np.zeros(n, np.uint32)
    nfr = int(np.frombuffer(s[20:24].tobytes(), np.uint32)[0]) if s.size >= 24 else 1
    kinds = np.zeros(max(nfr, 1), np.uint8)
    res = Result()
    rc = lib().nzo_decode_codes(_ptr(s), s.size, n, C.c_float(eb), _ptr(q), _ptr(rb), _ptr(kinds), C.byref(res))
    return q, rb, kinds, res, rc


def reduce_frames(a, b, n, eb, opts=None, cap=None):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    b = np.ascontiguousarray(b, dtype=np.uint8)
    if cap is None:
        cap = compress_bound(n, opts)
    out = np.zeros(max(cap, 1), np.uint8)
    res = Result()
    rc = lib().nzo_reduce_frames(_ptr(a), a.size, _ptr(b), b.size, _ptr(out), cap, n, C.c_float(eb),
                                 C.byref(opts) if opts is not None else None, C.byref(res))
    return out[:res.bytes].copy(), res, rc


def reduce_k(streams, n, eb, opts=None, cap=None, step=None):
    """k-ary reduce: one output stream from the operand streams, taken in the order given (step: the bin width of
    streams made by the stochastic quantizer, in the place of the error bound)."""
    arrs = [np.ascontiguousarray(s, dtype=np.uint8) for s in streams]
    k = len(arrs)
    ptrs = (C.c_void_p * max(k, 1))(*[a.ctypes.data for a in arrs])
    sizes = (C.c_size_t * max(k, 1))(*[a.size for a in arrs])
    if cap is None:
        cap = compress_bound(n, opts)
    out = np.zeros(max(cap, 1), np.uint8)
    res = Result()
    fn = lib().nzo_reduce_k if step is None else lib().nzo_reduce_k_step
    rc = fn(ptrs, sizes, k, _ptr(out), cap, n, C.c_float(eb if step is None else step),
            C.byref(opts) if opts is not None else None, C.byref(res))
    return out[:res.bytes].copy(), res, rc


def reduce_local(a, x, eb, opts=None, cap=None):
    """Ring-step reduce: incoming stream `a` plus the rank's own fp32 message `x` (quantized, never entropy coded)."""
    a = np.ascontiguousarray(a, dtype=np.uint8)
    x = np.ascontiguousarray(x, dtype=np.float32)
    n = x.size
    if cap is None:
        cap = compress_bound(n, opts)
    out = np.zeros(max(cap, 1), np.uint8)
    res = Result()
    rc = lib().nzo_reduce_local(_ptr(a), a.size, _ptr(x), _ptr(out), cap, n, C.c_float(eb),
                                C.byref(opts) if opts is not None else None, C.byref(res))
    return out[:res.bytes].copy(), res, rc


def frame_plan(q, opts=None, quantizable=True):
    """Plan one frame of integer codes.  Returns dict with the selector's choice and exact sizes."""
    q = np.ascontiguousarray(q, dtype=np.int32)
    K = (opts.alphabet if opts is not None and opts.alphabet else 256)
    totals = np.zeros(3, np.uint64)
    pay = np.zeros(3, np.uint64)
    w = np.zeros(1, np.uint32)
    nsym = np.zeros(1, np.uint32)
    hb = np.zeros(1, np.uint64)
    ln = np.zeros(K, np.uint8)
    code = np.zeros(K, np.uint32)
    c = lib().nzo_frame_plan(_ptr(q), q.size, int(bool(quantizable)), C.byref(opts) if opts is not None else None,
                             _ptr(totals), _ptr(pay), _ptr(w), _ptr(nsym), _ptr(hb), _ptr(ln), _ptr(code))
    if c < 0:
        raise ValueError("bad frame/opts")
    return dict(codec=c, totals=totals.astype(np.int64), payloads=pay.astype(np.int64), w=int(w[0]),
                nsym=int(nsym[0]), huff_bits=int(hb[0]), len=ln, code=code)


def frame_encode(q, codec, opts=None, step_bits=0, rawbits=None):
    q = np.ascontiguousarray(q, dtype=np.int32)
    if rawbits is None:
        rawbits = np.zeros(q.size, np.uint32)
    rawbits = np.ascontiguousarray(rawbits, dtype=np.uint32)
    cap = 64 + 8 * q.size + 4096
    dst = np.zeros(cap, np.uint8)
    t = lib().nzo_frame_encode(_ptr(q), _ptr(rawbits), q.size, codec, C.byref(opts) if opts is not None else None,
                               step_bits, _ptr(dst), cap)
    if t < 0:
        raise ValueError("frame_encode failed: %d" % t)
    return dst[:t].copy()


def context_build(sample, eb, opts=None):
    """Huffman context (cached codebook) from a calibration message of at most 2^20 values."""
    x = np.ascontiguousarray(sample, dtype=np.float32)
    ctx = Context()
    rc = lib().nzo_context_build(_ptr(x), x.size, C.c_float(eb), C.byref(opts) if opts is not None else None, C.byref(ctx))
    if rc:
        raise ValueError("context_build failed: %d" % rc)
    return ctx


def rea_plan_frame(x, eb, opts=None, ropts=None, ctx=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    P = ReaPlan()
    rc = lib().nzo_rea_plan_frame(_ptr(x), x.size, C.c_float(eb), C.byref(opts) if opts is not None else None,
                                  C.byref(ropts) if ropts is not None else None,
                                  C.byref(ctx) if ctx is not None else None, C.byref(P))
    if rc:
        raise ValueError("rea_plan_frame failed: %d" % rc)
    return dict(n_s=int(P.n_s), sample_ok=bool(P.sample_ok), w_s=int(P.w_s), sample_bits=int(P.sample_bits),
                pred_payload=[int(v) for v in P.pred_payload], plan=int(P.plan))


def compress_rea(x, eb, opts=None, ropts=None, ctx=None, cap=None):
    """Sampled arbitration (Algorithm 1).  Returns (slotted stream trimmed to its span, ReaResult, rc, planned codec
    per frame)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if cap is None:
        o = opts if opts is not None else make_opts()
        cap = compress_bound(x.size, make_opts(o.chunk_elems, o.seg_syms, o.alphabet, -1, 0, 0))
    out = np.zeros(max(cap, 1), np.uint8)
    res = ReaResult()
    chunk = (opts.chunk_elems if opts is not None and opts.chunk_elems else 262144)
    plans = np.zeros(max(1, (x.size + chunk - 1) // chunk), np.uint8)
    rc = lib().nzo_compress_rea(_ptr(x), x.size, C.c_float(eb), C.byref(opts) if opts is not None else None,
                                C.byref(ropts) if ropts is not None else None,
                                C.byref(ctx) if ctx is not None else None, _ptr(out), cap, C.byref(res), _ptr(plans))
    return out[:res.span_bytes].copy(), res, rc, plans


def reduce_local_rea(a, x, eb, opts=None, ropts=None, ctx=None, cap=None):
    """Ring-step reduce with the sampled arbitration on the way out.  Returns (slotted stream trimmed to its span,
    ReaResult, rc, planned codec per frame)."""
    a = np.ascontiguousarray(a, dtype=np.uint8)
    x = np.ascontiguousarray(x, dtype=np.float32)
    if cap is None:
        o = opts if opts is not None else make_opts()
        cap = compress_bound(x.size, make_opts(o.chunk_elems, o.seg_syms, o.alphabet, -1, 0, 0))
    out = np.zeros(max(cap, 1), np.uint8)
    res = ReaResult()
    chunk = (opts.chunk_elems if opts is not None and opts.chunk_elems else 262144)
    plans = np.zeros(max(1, (x.size + chunk - 1) // chunk), np.uint8)
    rc = lib().nzo_reduce_local_rea(_ptr(a), a.size, _ptr(x), x.size, C.c_float(eb), C.byref(opts) if opts is not None else None,
                                    C.byref(ropts) if ropts is not None else None,
                                    C.byref(ctx) if ctx is not None else None, _ptr(out), cap, C.byref(res), _ptr(plans))
    return out[:res.span_bytes].copy(), res, rc, plans


def sr_draw(seed, i):
    return int(lib().nzo_sr_draw(seed, i))


def sr_quantize(x, step, seed, first_index=0):
    """Stochastic (QSGD-style) rounding to multiples of step; element k uses draw (seed, first_index + k)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.size, np.int32)
    ok = np.empty(x.size, np.uint8)
    rc = lib().nzo_sr_quantize(_ptr(x), x.size, C.c_float(step), seed, first_index, _ptr(q), _ptr(ok))
    if rc:
        raise ValueError("invalid step")
    return q, ok.astype(bool)


def qsgd_step(x, levels):
    x = np.ascontiguousarray(x, dtype=np.float32)
    st = C.c_float()
    rc = lib().nzo_qsgd_step(_ptr(x), x.size, levels, C.byref(st))
    if rc:
        raise ValueError("qsgd_step failed: %d" % rc)
    return float(st.value)


def compress_sr(x, step, seed, opts=None, cap=None):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if cap is None:
        cap = compress_bound(x.size, opts)
    out = np.zeros(max(cap, 1), np.uint8)
    res = Result()
    rc = lib().nzo_compress_sr(_ptr(x), x.size, C.c_float(step), seed, C.byref(opts) if opts is not None else None,
                               _ptr(out), cap, C.byref(res))
    return out[:res.bytes].copy(), res, rc


def decompress_step(stream, n, step):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    out = np.zeros(n, np.float32)
    res = Result()
    rc = lib().nzo_decompress_step(_ptr(s), s.size, _ptr(out), n, C.c_float(step), C.byref(res))
    return out, res, rc


def decode_codes_step(stream, n, step):
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    q = np.zeros(n, np.int32)
    rb = np.zeros(n, np.uint32)
    nfr = int(np.frombuffer(s[20:24].tobytes(), np.uint32)[0]) if s.size >= 24 else 1
    kinds = np.zeros(max(nfr, 1), np.uint8)
    res = Result()
    rc = lib().nzo_decode_codes_step(_ptr(s), s.size, n, C.c_float(step), _ptr(q), _ptr(rb), _ptr(kinds), C.byref(res))
    return q, rb, kinds, res, rc


def reduce_local_sr(a, x, step, seed, opts=None, cap=None):
    """Ring-step reduce with the stochastic quantizer: incoming stream `a` plus the rank's own fp32 message `x`."""
    a = np.ascontiguousarray(a, dtype=np.uint8)
    x = np.ascontiguousarray(x, dtype=np.float32)
    n = x.size
    if cap is None:
        cap = compress_bound(n, opts)
    out = np.zeros(max(cap, 1), np.uint8)
    res = Result()
    rc = lib().nzo_reduce_local_sr(_ptr(a), a.size, _ptr(x), _ptr(out), cap, n, C.c_float(step), seed,
                                   C.byref(opts) if opts is not None else None, C.byref(res))
    return out[:res.bytes].copy(), res, rc


def reduce_frames_step(a, b, n, step, opts=None, cap=None):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    b = np.ascontiguousarray(b, dtype=np.uint8)
    if cap is None:
        cap = compress_bound(n, opts)
    out = np.zeros(max(cap, 1), np.uint8)
    res = Result()
    rc = lib().nzo_reduce_frames_step(_ptr(a), a.size, _ptr(b), b.size, _ptr(out), cap, n, C.c_float(step),
                                      C.byref(opts) if opts is not None else None, C.byref(res))
    return out[:res.bytes].copy(), res, rc
