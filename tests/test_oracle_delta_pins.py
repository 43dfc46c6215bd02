"""Pins of the oracle's delta predictor on the codes (an extension in front of the entropy stage: the prediction stage
of the SZ-style pipeline that Sec. II-B lists).  What fixes it: the predicted values are numpy's differences with a
restart at every segment, so the whole coded frame must equal the (separately pinned) plain frame of those
differences; the receiver's running sums give the codes back, also where differences wrap around 2^32; prediction
commutes with the integer reduce; smooth data gets smaller."""
import numpy as np
import pytest

import oracle
from paper_2605_12396_amd import workloads as W

EB1 = float(np.float32(32.0 / 63.0))          # step = 1 exactly: x = q


def _delta(q, seg):
    q = np.asarray(q, np.int64)
    d = q.copy()
    d[1:] -= q[:-1]
    d[::seg] = q[::seg]
    return (((d + 2 ** 31) % 2 ** 32) - 2 ** 31).astype(np.int32)       # modulo 2^32, as a signed value


@pytest.mark.parametrize("seg", [256, 64, 1000])
@pytest.mark.parametrize("K", [256, 1024, 16])
def test_delta_frame_is_the_plain_frame_of_the_differences(seg, K):
    rng = np.random.default_rng(seg + K)
    nf = 5000
    t = np.arange(nf)
    q = (3000 * np.sin(t / 150.0) + rng.integers(-3, 4, nf)).astype(np.int32)
    q[777] = 30000                                                    # a jump: the difference escapes
    od = oracle.make_opts(chunk_elems=nf, seg_syms=seg, alphabet=K, predictor=1)
    op = oracle.make_opts(chunk_elems=nf, seg_syms=seg, alphabet=K)
    d = _delta(q, seg)
    pd, pp = oracle.frame_plan(q, od), oracle.frame_plan(d, op)
    for k in ("codec", "w", "nsym", "huff_bits"):
        assert pd[k] == pp[k], k
    assert (pd["totals"] == pp["totals"]).all() and (pd["len"] == pp["len"]).all() and (pd["code"] == pp["code"]).all()
    for codec in (1, 2):
        fd = oracle.frame_encode(q, codec, od, step_bits=123)
        fp = oracle.frame_encode(d, codec, op, step_bits=123)
        hd, hp = fd[:32].view(np.uint32), fp[:32].view(np.uint32)
        assert (fd[32:] == fp[32:]).all() and (hd[:5] == hp[:5]).all() and hd[6] == hp[6]
        assert hd[5] == hp[5] | (1 << 31) and hd[7] == hp[7] ^ (1 << 31)      # the flag and the check word over it
    # much smaller than coding the codes themselves on a smooth signal
    if K >= 256:
        assert pd["totals"][2] < 0.6 * oracle.frame_plan(q, op)["totals"][2]


def test_roundtrip_values_bound_and_ratio_on_smooth_data():
    n = 200000
    x = (np.sin(np.arange(n) / 300.0) + 1e-4 * np.random.default_rng(1).normal(size=n)).astype(np.float32)
    eb = 1e-4
    for kw in (dict(chunk_elems=65536), dict(chunk_elems=20000, alphabet=1024), dict(chunk_elems=10003, seg_syms=100)):
        od, op = oracle.make_opts(predictor=1, **kw), oracle.make_opts(**kw)
        sd, rd, rc = oracle.compress(x, eb, od)
        sp, rp, rc2 = oracle.compress(x, eb, op)
        assert rc == 0 and rc2 == 0 and int(sd[36:40].view(np.uint32)[0]) == 1 and int(sp[36:40].view(np.uint32)[0]) == 0
        assert sd.size < 0.5 * sp.size
        q, ok = oracle.quantize(x, eb)
        qd, rb, kinds, res, drc = oracle.decode_codes(sd, n, eb)
        assert drc == 0 and not kinds.any() and (qd == q).all()
        yd, yp = oracle.decompress(sd, n, eb)[0], oracle.decompress(sp, n, eb)[0]
        assert (yd.view(np.uint32) == yp.view(np.uint32)).all()
        assert (np.abs(yd.astype(np.float64) - x) <= np.float32(eb)).all()
    # white noise gets slightly larger (the difference of two independent codes has twice the variance)
    g = W.gradient_like(100000, seed=3, outlier_frac=0.0)
    a = oracle.compress(g, 1e-4, oracle.make_opts(chunk_elems=50000, predictor=1))[0].size
    b = oracle.compress(g, 1e-4, oracle.make_opts(chunk_elems=50000))[0].size
    assert b < a < 1.25 * b
    # a frame that cannot be quantized is RAW as before
    z = x.copy(); z[70000] = np.nan
    s, r, rc = oracle.compress(z, eb, oracle.make_opts(chunk_elems=65536, predictor=1))
    assert rc == 0 and r.n_raw == 1
    out = oracle.decompress(s, n, eb)[0]
    assert (out[65536:131072].view(np.uint32) == z[65536:131072].view(np.uint32)).all()


def test_prediction_commutes_with_the_integer_reduce_and_wraps_modulo_2_32():
    n, eb = 3000, 1e-3
    od = oracle.make_opts(chunk_elems=1000, predictor=1)
    a = (np.sin(np.arange(n) / 40.0) * 0.5).astype(np.float32)
    b = (np.cos(np.arange(n) / 25.0) * 0.3).astype(np.float32)
    sa, sb = oracle.compress(a, eb, od)[0], oracle.compress(b, eb, od)[0]
    qa, qb = oracle.quantize(a, eb)[0], oracle.quantize(b, eb)[0]
    red, res, rc = oracle.reduce_frames(sa, sb, n, eb, od)
    assert rc == 0 and (oracle.decode_codes(red, n, eb)[0] == qa + qb).all()
    step_bits = int(np.float32(oracle.step_constants(eb)[0]).view(np.uint32))
    offs = red[64:64 + 24].view(np.uint64).astype(np.int64)
    for k in range(3):
        qs = (qa + qb)[k * 1000:(k + 1) * 1000]
        fr = oracle.frame_encode(qs, oracle.frame_plan(qs, od)["codec"], od, step_bits=step_bits)
        assert (red[offs[k]:offs[k] + fr.size] == fr).all()
    assert oracle.reduce_frames(sb, sa, n, eb, od)[0].tobytes() == red.tobytes()
    lo, lres, lrc = oracle.reduce_local(sa, b, eb, od)
    assert lrc == 0 and lo.tobytes() == red.tobytes()
    # operands and options must agree on the predictor
    op = oracle.make_opts(chunk_elems=1000)
    assert oracle.reduce_frames(sa, sb, n, eb, op)[2] == oracle.ERR_MISMATCH
    assert oracle.reduce_frames(sa, oracle.compress(b, eb, op)[0], n, eb, od)[2] == oracle.ERR_MISMATCH
    assert oracle.reduce_local(oracle.compress(a, eb, op)[0], b, eb, od)[2] == oracle.ERR_MISMATCH
    # codes +2^30 next to -2^30: the difference is -2^31 (and +2^31, which wraps to -2^31); sums come back exactly
    y = np.zeros(1000, np.float32); step = oracle.step_constants(eb)[0]
    y[3], y[4], y[5] = step, -step, step
    t = oracle.compress(y, eb, od)[0]
    for _ in range(30):
        t = oracle.reduce_frames(t, t, 1000, eb, od)[0]
    q = oracle.decode_codes(t, 1000, eb)[0]
    assert q[[2, 3, 4, 5, 6]].tolist() == [0, 1 << 30, -(1 << 30), 1 << 30, 0]
    fr = oracle.frame_plan(q, od)
    assert fr["w"] == 32                                         # zigzag of -2^31 needs all 32 bits


def test_flags_are_validated_and_other_paths_refuse_the_predictor():
    n, eb = 5000, 1e-4
    x = W.gradient_like(n, seed=4)
    od = oracle.make_opts(chunk_elems=2000, predictor=1)
    s = oracle.compress(x, eb, od)[0]
    t = s.copy(); t[36] = 0                                      # stream says "no predictor", frames say delta
    assert oracle.decompress(t, n, eb)[2] == oracle.ERR_CORRUPT
    t = s.copy(); t[36] = 2
    assert oracle.decompress(t, n, eb)[2] == oracle.ERR_CORRUPT
    off = int(s[64:72].view(np.uint64)[0])
    t = s.copy(); t[off + 23] ^= 0x80; t[off + 31] ^= 0x80       # clear the frame's flag and fix the check word
    assert oracle.decompress(t, n, eb)[2] == oracle.ERR_CORRUPT
    with pytest.raises(ValueError):
        oracle.frame_plan(np.zeros(10, np.int32), oracle.make_opts(predictor=2))
    ctx = oracle.context_build(x, eb, oracle.make_opts())
    assert oracle.compress_rea(x, eb, od, None, ctx, cap=1 << 20)[2] == oracle.ERR_INVALID
    assert oracle.compress_sr(x, 1e-4, 1, od)[2] == oracle.ERR_INVALID
