"""Pins of the oracle's stochastic interface quantizer (QSGD: Sec. II-B "Quantization", Sec. IV-B) against things
other than itself: published values of the hash finalizer behind the counter-based draw, the two-neighbour rule,
rounding probabilities and unbiasedness by statistics, QSGD's variance bound, the norm-based bin width against numpy,
and the usual frame machinery (the stream of codes is coded like any other)."""
import math

import numpy as np
import pytest

import oracle
from paper_2605_12396_amd import workloads as W


def _fmix32(h):
    h &= 0xFFFFFFFF
    h ^= h >> 16; h = (h * 0x85EBCA6B) & 0xFFFFFFFF
    h ^= h >> 13; h = (h * 0xC2B2AE35) & 0xFFFFFFFF
    h ^= h >> 16
    return h


def test_draw_is_the_published_finalizer_keyed_by_seed_and_index():
    # values of MurmurHash3's 32-bit finalizer that circulate with the algorithm: fmix32(1), fmix32(0xFFFFFFFF)
    assert _fmix32(1) == 0x514E28B7 and _fmix32(0xFFFFFFFF) == 0x81F16F39 and _fmix32(0) == 0
    # seed 0 keys with fmix32(0) = 0, so the draw of element i < 2^32 is the top 24 bits of fmix32(i)
    assert oracle.sr_draw(0, 1) == 0x514E28 and oracle.sr_draw(0, 0xFFFFFFFF) == 0x81F16F and oracle.sr_draw(0, 0) == 0
    rng = np.random.default_rng(1)
    for _ in range(200):
        seed = int(rng.integers(0, 1 << 32)); i = int(rng.integers(0, 1 << 40))
        key = _fmix32((seed + 0x9E3779B9 * (i >> 32)) & 0xFFFFFFFF)
        assert oracle.sr_draw(seed, i) == _fmix32((i & 0xFFFFFFFF) ^ key) >> 8
    # 24-bit draws, roughly uniform
    d = np.array([oracle.sr_draw(7, i) for i in range(20000)])
    assert d.max() < 1 << 24 and abs(d.mean() / 2 ** 24 - 0.5) < 0.01 and len(set(d.tolist())) > 19900


def test_two_neighbour_rule_grid_points_and_sign():
    step = 0.25                                             # exact in binary: a = |x| / step has no rounding
    x = np.array([0.0, 0.25, -0.25, 1.0, -8191.75, 0.3, -0.3, 0.49, 100.1], np.float32)
    for seed in range(50):
        q, ok = oracle.sr_quantize(x, step, seed)
        assert ok.all()
        a = np.abs(x.astype(np.float64)) / step
        lo = np.floor(a)
        mag = np.abs(q)
        assert ((mag == lo) | (mag == lo + 1)).all()
        assert (np.sign(q) == np.sign(x) * (mag > 0)).all()
        assert q[:5].tolist() == [0, 1, -1, 4, -32767]       # grid points never move
    # element k of a message uses draw (seed, k): quantizing a tail with first_index = k gives the same codes
    y = W.gradient_like(5000, seed=3)
    q_all, _ = oracle.sr_quantize(y, 1e-4, 11)
    q_tail, _ = oracle.sr_quantize(y[1234:], 1e-4, 11, first_index=1234)
    assert (q_all[1234:] == q_tail).all()
    assert (oracle.sr_quantize(y, 1e-4, 12)[0] != q_all).any()
    # the high half of a 64-bit index takes part in the draw
    assert (oracle.sr_quantize(y[:500], 1e-4, 5, first_index=(1 << 33) + 7)[0] != oracle.sr_quantize(y[:500], 1e-4, 5, first_index=7)[0]).any()


def test_rounding_probability_and_unbiasedness():
    step = 0.5
    N = 200000
    for frac in (0.0, 0.1, 0.5, 0.9, 1.0 / 3.0):
        x = np.full(N, (3 + frac) * step, np.float32)
        a = float(x[0]) / step
        f = a - math.floor(a)
        q, ok = oracle.sr_quantize(x, step, 99)
        assert ok.all() and set(q.tolist()) <= {3, 4}
        p_up = (q == 4).mean()
        assert abs(p_up - f) <= 5 * math.sqrt(max(f * (1 - f), 1e-9) / N) + 2.0 ** -23
    # unbiased on a whole message: E[q * step] = x
    x = W.gradient_like(200000, seed=4, outlier_frac=0.0)
    step = oracle.qsgd_step(x, 16)
    xh = np.zeros(x.size, np.float64)
    S = 64
    for seed in range(S):
        q, ok = oracle.sr_quantize(x, step, seed)
        xh += q.astype(np.float64) * step
    xh /= S
    # per element the estimator has variance <= step^2 / 4; the mean over all elements of (xh - x) must vanish
    assert abs((xh - x).mean()) < 5 * (step / 2) / math.sqrt(S * x.size)
    assert np.abs(xh - x).max() < 6 * (step / 2) / math.sqrt(S) + 1e-9


def test_qsgd_step_levels_and_variance_bound():
    x = W.gradient_like(100000, seed=5)
    for s in (1, 4, 256, 32767):
        step = oracle.qsgd_step(x, s)
        ref = math.sqrt(float((x.astype(np.float64) ** 2).sum())) / s
        assert abs(step - ref) <= 2.0 ** -23 * ref
        q, ok = oracle.sr_quantize(x, step, 3)
        assert ok.all() and np.abs(q).max() <= s               # |x_i| <= ||x||_2: never more than s levels
    # QSGD's second-moment bound: E||Q(v) - v||^2 <= min(n / s^2, sqrt(n) / s) ||v||^2
    n, s = 4096, 16
    v = np.random.default_rng(6).normal(0, 1, n).astype(np.float32)
    step = oracle.qsgd_step(v, s)
    err = np.mean([((oracle.sr_quantize(v, step, seed)[0] * np.float64(step) - v) ** 2).sum() for seed in range(40)])
    assert err <= min(n / s ** 2, math.sqrt(n) / s) * float((v.astype(np.float64) ** 2).sum())
    assert oracle.qsgd_step(np.zeros(10, np.float32), 8) == 2.0 ** -100
    with pytest.raises(ValueError):
        oracle.qsgd_step(x, 0)
    with pytest.raises(ValueError):
        oracle.qsgd_step(np.array([np.inf, 1.0], np.float32), 8)


def test_error_and_range():
    rng = np.random.default_rng(7)
    for step in (1e-4, 0.37, 3.0e-30, 5e20):
        x = (rng.uniform(-1, 1, 200000) * 32700 * step).astype(np.float32)
        q, ok = oracle.sr_quantize(x, np.float32(step), 21)
        st = float(np.float32(step))
        assert ok.all()
        err = np.abs(x.astype(np.float64) - q.astype(np.float64) * st)
        assert (err <= st * (1 + 2.0 ** -6)).all()
    x = np.array([np.nan, np.inf, -np.inf, 32768.5, -40000.0, 32766.0], np.float32)
    q, ok = oracle.sr_quantize(x, 1.0, 1)
    assert ok.tolist() == [False, False, False, False, False, True]


def test_stream_is_the_coded_stochastic_codes_and_reduces_exactly():
    n = 3 * 20000 + 777
    x, y = W.gradient_like(n, seed=8), W.gradient_like(n, seed=9)
    o = oracle.make_opts(chunk_elems=20000)
    step = max(oracle.qsgd_step(x, 256), oracle.qsgd_step(y, 256))       # ranks that reduce share one width
    sx, rx, rc = oracle.compress_sr(x, step, 5, o)
    sy, ry, rc2 = oracle.compress_sr(y, step, 6, o)
    assert rc == 0 and rc2 == 0 and int(sx[24:28].view(np.uint32)[0]) == int(np.float32(step).view(np.uint32))
    qx, okx = oracle.sr_quantize(x, step, 5); qy, oky = oracle.sr_quantize(y, step, 6)
    assert okx.all() and oky.all()
    qd, rb, kinds, res, drc = oracle.decode_codes_step(sx, n, step)
    assert drc == 0 and not kinds.any() and (qd == qx).all()
    # every frame is exactly what the frame encoder makes of those codes under the selector's choice
    step_bits = int(np.float32(step).view(np.uint32))
    offs = sx[64:64 + 8 * 4].view(np.uint64).astype(np.int64)
    for k in range(4):
        qf = qx[k * 20000:(k + 1) * 20000]
        plan = oracle.frame_plan(qf, o)
        fr = oracle.frame_encode(qf, plan["codec"], o, step_bits=step_bits)
        assert (sx[offs[k]:offs[k] + fr.size] == fr).all()
    out, dres, drc = oracle.decompress_step(sx, n, step)
    assert drc == 0 and (out == (qx.astype(np.float32) * np.float32(step)).astype(np.float32)).all()
    assert oracle.decompress_step(sx, n, np.float32(step) * 2)[2] == oracle.ERR_MISMATCH
    red, rres, rrc = oracle.reduce_frames_step(sx, sy, n, step, o)
    assert rrc == 0 and (oracle.decode_codes_step(red, n, step)[0] == qx + qy).all()
    # a value that cannot be quantized turns its frame RAW, as with the deterministic quantizer
    z = x.copy(); z[25000] = np.nan
    sz, rz, rc = oracle.compress_sr(z, step, 5, o)
    assert rc == 0 and rz.n_raw == 1
    outz = oracle.decompress_step(sz, n, step)[0]
    assert (outz[20000:40000].view(np.uint32) == z[20000:40000].view(np.uint32)).all()


def test_ring_step_with_the_stochastic_quantizer():
    """nzo_reduce_local_sr(in, x) must be, byte for byte, the two-stream reduce of `in` with the stochastic stream of x
    (same seed), its codes the exact sums of the incoming codes and the drawn codes, and its special frames (incoming
    RAW, local value that cannot be quantized, sums past 2^30) must follow the same rules."""
    n = 70001
    o = oracle.make_opts(chunk_elems=20000)
    a, x = W.gradient_like(n, seed=61), W.gradient_like(n, seed=62)
    step = float(np.float32(max(oracle.qsgd_step(a, 128), oracle.qsgd_step(x, 128))))
    sa, _, rc = oracle.compress_sr(a, step, 11, o)
    sx, _, rc2 = oracle.compress_sr(x, step, 12, o)
    two, tres, rc3 = oracle.reduce_frames_step(sa, sx, n, step, o)
    one, ores, rc4 = oracle.reduce_local_sr(sa, x, step, 12, o)
    assert rc == 0 and rc2 == 0 and rc3 == 0 and rc4 == 0 and one.size == two.size and (one == two).all()
    qa, _ = oracle.sr_quantize(a, step, 11)
    qx, _ = oracle.sr_quantize(x, step, 12)
    q, rb, kinds, _, drc = oracle.decode_codes_step(one, n, step)
    assert drc == 0 and not kinds.any() and (q == qa + qx).all()
    # another seed gives another stream; the deterministic ring step too
    assert not np.array_equal(oracle.reduce_local_sr(sa, x, step, 13, o)[0], one)
    # incoming RAW frame, local frame with a value that cannot be quantized
    a2, x2 = a.copy(), x.copy()
    a2[5] = np.inf; x2[45000] = np.nan
    sa2, _, _ = oracle.compress_sr(a2, step, 11, o)
    sx2, _, _ = oracle.compress_sr(x2, step, 12, o)
    one2, r2, rc5 = oracle.reduce_local_sr(sa2, x2, step, 12, o)
    two2, _, _ = oracle.reduce_frames_step(sa2, sx2, n, step, o)
    assert rc5 == 0 and r2.n_raw == 2 and (one2 == two2).all()
    y, _, _ = oracle.decompress_step(one2, n, step)
    st = np.float32(step)
    assert np.isinf(y[5]) and np.isnan(y[45000])
    assert y[6] == np.float32(a2[6] + np.float32(np.float32(qx[6]) * st))               # raw incoming value + local code
    assert y[45001] == np.float32(np.float32(np.float32(qa[45001]) * st) + x2[45001])   # incoming code + original local value
    # mismatches and refusals
    assert oracle.reduce_local_sr(sa, x, step * 2, 12, o)[2] == oracle.ERR_MISMATCH
    assert oracle.reduce_local_sr(sa, x[:-1], step, 12, o)[2] == oracle.ERR_MISMATCH
    assert oracle.reduce_local_sr(sa, x, step, 12, oracle.make_opts(chunk_elems=20000, predictor=1))[2] == oracle.ERR_INVALID
    assert oracle.reduce_local_sr(sa, x, 0.0, 12, o)[2] == oracle.ERR_INVALID
