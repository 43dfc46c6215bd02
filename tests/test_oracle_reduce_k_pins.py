"""Pins of the oracle's k-ary reduce (the reduction of Sec. IV-D "In-Primitive Overlap" over all the contributions a
rank holds at once) against things other than itself: the chain of the separately pinned two-operand reduce byte for
byte, numpy sums of the separately decoded codes, numpy's fp32 left fold where a frame leaves the integer domain
(RAW operand, partial sum beyond 2^30), order independence of integer sums, the k-fold error bound, refusals."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2605_12396_amd import workloads as W


def _chain(streams, n, eb, opts):
    acc = streams[0]
    for s in streams[1:]:
        acc, res, rc = oracle.reduce_frames(acc, s, n, eb, opts)
        assert rc == 0
    return acc


@pytest.mark.parametrize("k", [2, 3, 5, 8])
@pytest.mark.parametrize("kw", [dict(), dict(alphabet=1024), dict(predictor=1), dict(force_codec=1), dict(force_codec=2)])
def test_equals_the_chain_of_two_operand_reduces(k, kw):
    n, eb = 5000 + 37 * k, 1e-4
    opts = oracle.make_opts(chunk_elems=1024, **kw)
    xs = [W.gradient_like(n, seed=300 + p, b=1e-3 * (1 + p % 3)) for p in range(k)]
    ss = [oracle.compress(x, eb, opts)[0] for x in xs]
    r, res, rc = oracle.reduce_k(ss, n, eb, opts)
    assert rc == 0 and res.status == 0 and res.bytes == r.size
    assert np.array_equal(r, _chain(ss, n, eb, opts))
    # the codes are the numpy sum of the separately decoded codes
    q = sum(oracle.decode_codes(s, n, eb)[0].astype(np.int64) for s in ss)
    qd, _, kinds, _, _ = oracle.decode_codes(r, n, eb)
    assert not kinds.any() and (qd == q).all()
    # and the k-fold bound holds against the float64 sum of the inputs
    out = oracle.decompress(r, n, eb)[0]
    exact = np.sum(np.stack([x.astype(np.float64) for x in xs]), axis=0)
    assert np.abs(out.astype(np.float64) - exact).max() <= k * eb * (1 + 1e-6)


@pytest.mark.parametrize("k", [2, 3, 6])
@pytest.mark.parametrize("kw", [dict(min_gain_permil=700), dict(force_codec=0), dict(huff_min_bytes=1 << 20, min_gain_permil=600)])
def test_options_that_turn_integer_sums_raw_apply_to_the_final_stream_only(k, kw):
    # the operands are summed as codes whatever the options say; the selector sees the final sums, and a frame it
    # commits RAW holds the fp32 form of the last step -- exactly the two-operand reduce of (all but the last, the last)
    n, eb = 4100, 1e-4
    plain = oracle.make_opts(chunk_elems=1024)
    gated = oracle.make_opts(chunk_elems=1024, **kw)
    xs = [W.gradient_like(n, seed=310 + p, b=1e-3 * (1 + p % 2)) for p in range(k)]
    ss = [oracle.compress(x, eb, plain)[0] for x in xs]
    r, res, rc = oracle.reduce_k(ss, n, eb, gated)
    assert rc == 0 and res.n_raw > 0
    head = ss[0] if k == 2 else oracle.reduce_k(ss[:-1], n, eb, plain)[0]
    want, wres, wrc = oracle.reduce_frames(head, ss[-1], n, eb, gated)
    assert wrc == 0 and np.array_equal(r, want)
    # a RAW frame of integer sums decodes to numpy's fp32 sum of the two dequantized operands of the last step
    out = oracle.decompress(r, n, eb)[0]
    kinds = oracle.decode_codes(r, n, eb)[2]
    fp = (oracle.decompress(head, n, eb)[0] + oracle.decompress(ss[-1], n, eb)[0]).astype(np.float32)
    for f in np.nonzero(kinds)[0]:
        assert np.array_equal(out[1024 * f:1024 * (f + 1)], fp[1024 * f:1024 * (f + 1)])


def test_integer_sums_do_not_depend_on_the_order():
    n, eb = 4000, 1e-4
    opts = oracle.make_opts(chunk_elems=1000)
    ss = [oracle.compress(W.gradient_like(n, seed=320 + p), eb, opts)[0] for p in range(4)]
    ref = oracle.reduce_k(ss, n, eb, opts)[0]
    for perm in itertools.permutations(range(4)):
        assert np.array_equal(oracle.reduce_k([ss[i] for i in perm], n, eb, opts)[0], ref)


def test_raw_operand_in_the_middle_is_numpys_fp32_left_fold():
    n, eb = 3000, 1e-3
    opts = oracle.make_opts(chunk_elems=1000)
    step, _ = oracle.step_constants(eb)
    xs = [W.gradient_like(n, seed=330 + p) for p in range(4)]
    xs[2][1500] = np.nan; xs[2][1501] = 3e30                    # frame 1 of operand 2 is RAW
    xs[0][2500] = -np.inf                                       # frame 2 of operand 0 is RAW from the start
    ss = [oracle.compress(x, eb, opts)[0] for x in xs]
    r, res, rc = oracle.reduce_k(ss, n, eb, opts)
    assert rc == 0 and (res.n_raw, res.n_frames) == (2, 3)
    assert np.array_equal(r, _chain(ss, n, eb, opts))
    qs = [oracle.decode_codes(s, n, eb)[0] for s in ss]
    ds = [oracle.decompress(s, n, eb)[0] for s in ss]
    qd, rb, kinds, _, _ = oracle.decode_codes(r, n, eb)
    assert kinds.tolist() == [0, 1, 1]
    assert (qd[:1000] == qs[0][:1000] + qs[1][:1000] + qs[2][:1000] + qs[3][:1000]).all()
    with np.errstate(invalid="ignore", over="ignore"):
        # frame 1: integer codes for operands 0 + 1, fp32 from operand 2 on
        v = ((qs[0][1000:2000] + qs[1][1000:2000]).astype(np.float32) * np.float32(step)).astype(np.float32)
        v = (v + ds[2][1000:2000]).astype(np.float32)
        v = (v + ds[3][1000:2000]).astype(np.float32)
        # frame 2: fp32 all the way, in the order of the operands
        u = ds[0][2000:]
        for p in (1, 2, 3):
            u = (u + ds[p][2000:]).astype(np.float32)
    for got, want in ((rb[1000:2000], v), (rb[2000:], u)):
        bits = want.view(np.uint32).copy()
        bits[np.isnan(want)] = 0x7FC00000
        assert (got == bits).all()
    # with the RAW operand last the codes are added first: another grouping of the fp32 sum
    r2 = oracle.reduce_k([ss[0], ss[1], ss[3], ss[2]], n, eb, opts)[0]
    qd2, rb2, _, _, _ = oracle.decode_codes(r2, n, eb)
    with np.errstate(invalid="ignore", over="ignore"):
        v2 = ((qs[0][1000:2000] + qs[1][1000:2000] + qs[3][1000:2000]).astype(np.float32) * np.float32(step)).astype(np.float32)
        v2 = (v2 + ds[2][1000:2000]).astype(np.float32)
    bits = v2.view(np.uint32).copy(); bits[np.isnan(v2)] = 0x7FC00000
    assert (rb2[1000:2000] == bits).all()


def test_partial_sum_beyond_two_to_thirty_turns_the_frame_raw_at_that_operand():
    n, eb = 2000, 1e-3
    opts = oracle.make_opts(chunk_elems=1000)
    step, _ = oracle.step_constants(eb)
    y = np.zeros(n, np.float32); y[3] = step; y[4] = -step                        # codes +1, -1
    t = oracle.compress(y, eb, opts)[0]
    for _ in range(29):
        t = oracle.reduce_frames(t, t, n, eb, opts)[0]                            # codes +-2^29
    w = np.zeros(n, np.float32); w[3] = step; w[1500] = 5 * step                  # codes +1 (frame 0), +5 (frame 1)
    small = oracle.compress(w, eb, opts)[0]
    z = oracle.compress(np.zeros(n, np.float32), eb, opts)[0]
    # 2^29 + 2^29 = 2^30 is still a code; one more unit is not
    r, res, rc = oracle.reduce_k([t, t, z], n, eb, opts)
    assert rc == 0 and res.n_raw == 0 and oracle.decode_codes(r, n, eb)[0][3] == 1 << 30
    r, res, rc = oracle.reduce_k([t, t, small, t], n, eb, opts)
    assert rc == 0 and (res.n_raw, res.n_frames) == (1, 2)
    assert np.array_equal(r, _chain([t, t, small, t], n, eb, opts))
    qd, rb, kinds, _, _ = oracle.decode_codes(r, n, eb)
    assert kinds.tolist() == [1, 0] and qd[1500] == 5                             # the other frame stays integer
    f = np.float32
    v3 = f(f(f(1 << 30) * f(step)) + f(f(1) * f(step)))                           # the operand at which the sum left the range
    v3 = f(v3 + f(f(1 << 29) * f(step)))                                          # and the one after it, in fp32
    v4 = f(f(f(-(1 << 30)) * f(step)) + f(0.0)); v4 = f(v4 + f(f(-(1 << 29)) * f(step)))
    assert rb[3] == np.array([v3], np.float32).view(np.uint32)[0]
    assert rb[4] == np.array([v4], np.float32).view(np.uint32)[0]
    assert not rb[5:1000].any()
    # the same operands in an order whose partial sums stay in range until the end: overflow at the last operand
    r2 = oracle.reduce_k([small, t, t, t], n, eb, opts)[0]
    assert np.array_equal(r2, _chain([small, t, t, t], n, eb, opts))
    rb2 = oracle.decode_codes(r2, n, eb)[1]
    w3 = f(f(f((1 << 30) + 1) * f(step)) + f(f(1 << 29) * f(step)))
    assert rb2[3] == np.array([w3], np.float32).view(np.uint32)[0]


def test_refusals():
    n, eb = 3000, 1e-4
    opts = oracle.make_opts(chunk_elems=1000)
    xs = [W.gradient_like(n, seed=340 + p) for p in range(3)]
    ss = [oracle.compress(x, eb, opts)[0] for x in xs]
    assert oracle.reduce_k(ss[:1], n, eb, opts)[2] == oracle.ERR_INVALID
    assert oracle.reduce_k([ss[0]] * 65, n, eb, opts)[2] == oracle.ERR_INVALID
    assert oracle.reduce_k([ss[0]] * 64, n, eb, opts)[2] == 0
    # every operand must match n, frame size, bin width and predictor
    other = [oracle.compress(xs[1], 2e-4, opts)[0],
             oracle.compress(xs[1], eb, oracle.make_opts(chunk_elems=1500))[0],
             oracle.compress(xs[1][:2999], eb, opts)[0],
             oracle.compress(xs[1], eb, oracle.make_opts(chunk_elems=1000, predictor=1))[0]]
    for bad in other:
        for pos in range(3):
            ops = list(ss); ops[pos] = bad
            r, res, rc = oracle.reduce_k(ops, n, eb, opts)
            assert rc == oracle.ERR_MISMATCH and res.status == oracle.ERR_MISMATCH and res.bytes == 0
    # a damaged operand fails the call whatever its position
    for pos in range(3):
        bad = ss[pos].copy()
        off = int(bad[64:72].view(np.uint64)[0])
        bad[off + 28] ^= 0x10                                    # check word of frame 0
        ops = list(ss); ops[pos] = bad
        r, res, rc = oracle.reduce_k(ops, n, eb, opts)
        assert rc == oracle.ERR_CORRUPT and res.bytes == 0
        ops[pos] = ss[pos][:100]
        assert oracle.reduce_k(ops, n, eb, opts)[2] == oracle.ERR_CORRUPT
    # capacity: one byte short of the result
    r, res, rc = oracle.reduce_k(ss, n, eb, opts)
    assert rc == 0
    r2, res2, rc2 = oracle.reduce_k(ss, n, eb, opts, cap=r.size - 1)
    assert rc2 == oracle.ERR_CAPACITY and res2.bytes == 0
    assert np.array_equal(oracle.reduce_k(ss, n, eb, opts, cap=r.size)[0], r)


def test_streams_of_the_stochastic_quantizer_reduce_by_their_bin_width():
    # the *_step form is the same fold on streams that record a width instead of a bound: the chain of the pinned
    # two-operand *_step reduce byte for byte, and the sum of the drawn codes
    n = 5000
    opts = oracle.make_opts(chunk_elems=1024)
    xs = [W.gradient_like(n, seed=350 + p) for p in range(4)]
    step = float(np.float32(max(oracle.qsgd_step(x, 100) for x in xs)))
    ss = [oracle.compress_sr(x, step, 10 + p, opts)[0] for p, x in enumerate(xs)]
    r, res, rc = oracle.reduce_k(ss, n, None, opts, step=step)
    assert rc == 0
    acc = ss[0]
    for s2 in ss[1:]:
        acc = oracle.reduce_frames_step(acc, s2, n, step, opts)[0]
    assert np.array_equal(r, acc)
    q = sum(oracle.sr_quantize(x, step, 10 + p)[0].astype(np.int64) for p, x in enumerate(xs))
    assert (oracle.decode_codes_step(r, n, step)[0] == q).all()
    assert oracle.reduce_k(ss, n, None, opts, step=step * 2)[2] == oracle.ERR_MISMATCH
    assert oracle.reduce_k(ss, n, None, opts, step=float("nan"))[2] == oracle.ERR_INVALID
