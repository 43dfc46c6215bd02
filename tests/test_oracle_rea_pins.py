"""Pins of the oracle's sampled runtime entropy arbitration (Sec. IV-C, Eq. 1-2, Algorithm 1) against things other
than itself: hand-computed plans, brute force over the realized frames, Huffman optimality, closed-form sizes, the
unchanged decoder, and the fallback rules of Algorithm 1 (AcceptRealized / CommitRawOrFail)."""
import heapq

import numpy as np
import pytest

import oracle
from paper_2605_12396_amd import workloads as W

EB1 = float(np.float32(32.0 / 63.0))          # step = 1 exactly: x = q


def _unzig(z):
    z = np.asarray(z, np.int64)
    return ((z >> 1) ^ -(z & 1)).astype(np.float32)


def _frames(stream):
    """(offset, codec, payload bytes, padded total) of every frame, read from the container by hand."""
    nfr = int(stream[20:24].view(np.uint32)[0])
    offs = stream[64:64 + 8 * nfr].view(np.uint64).astype(np.int64)
    out = []
    for off in offs:
        h = stream[off:off + 32].view(np.uint32)
        out.append((int(off), int(h[1]), int(h[3]), (32 + int(h[3]) + 15) // 16 * 16))
    return out


def _heap_cost(f):
    h = [int(v) for v in f if v > 0]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def test_context_hand_computed_and_invariants():
    # K = 4 (escape + zigzag codes 0, 1, 2); calibration counts 5, 2, 1 -> counts + 1 = [1, 6, 3, 2] for symbols 0..3.
    # Two-queue merge by hand: (1, s0) + (2, s3) = 3; leaf (3, s2) wins the tie against that node: 3 + 3 = 6; leaf
    # (6, s1) wins the tie against that node: 6 + 6 = 12.  Depths: s1 = 1, s2 = 2, s0 = s3 = 3.
    cal = _unzig([0] * 5 + [1] * 2 + [2])
    o = oracle.make_opts(alphabet=4)
    ctx = oracle.context_build(cal, EB1, o)
    assert ctx.valid == 1 and ctx.K == 4 and list(ctx.len[:4]) == [3, 1, 2, 3]
    assert list(ctx.code[:4]) == [0b110, 0b0, 0b10, 0b111]                  # canonical: (length, symbol) order
    # general: every symbol owns a code, Kraft sum exactly 1, optimal for (histogram + 1), canonical
    for seed, K in ((1, 256), (2, 1024), (3, 16)):
        x = W.gradient_like(50000, seed=seed)
        eb = 1e-4
        ok = oracle.make_opts(alphabet=K)
        ctx = oracle.context_build(x, eb, ok)
        ln = np.array(ctx.len[:K], np.int64)
        assert ln.min() >= 1 and ln.max() <= 28 and sum(2.0 ** -l for l in ln) == 1.0
        q, qok = oracle.quantize(x, eb)
        z = ((q.astype(np.int64) << 1) ^ (q.astype(np.int64) >> 31))[qok]
        f = np.bincount(np.where(z <= K - 2, z + 1, 0), minlength=K) + 1
        assert int((f * ln).sum()) == _heap_cost(f)
        assert (oracle.canonical_codes(ln.astype(np.uint8)) == np.array(ctx.code[:K])).all()
    with pytest.raises(ValueError):
        oracle.context_build(np.zeros((1 << 20) + 1, np.float32), 1e-4)


def test_plan_hand_computed_sizes_and_tie():
    """K = 4 context of the test above; a 10-element frame with a 16-byte sample window (4 elements, zigzag 0,0,1,2):
    sample bits = 1 + 1 + 2 + 3 = 7, predicted bits = ceil(7 * 10 / 4) = 18, HUFFMAN payload = 4 (lengths) + 4 (one
    segment entry, padded) + 4 = 12; FIXEDLEN width 2: 4 * ceil(20 / 32) = 4; RAW 40.  Totals pad16(32 + p): 48 for
    both coded paths -- the tie goes to the lower codec id, FIXEDLEN."""
    o = oracle.make_opts(chunk_elems=10, alphabet=4)
    ctx = oracle.context_build(_unzig([0] * 5 + [1] * 2 + [2]), EB1, o)
    x = _unzig([0, 0, 1, 2, 2, 1, 0, 0, 1, 0])
    P = oracle.rea_plan_frame(x, EB1, o, oracle.ReaOpts(16, 0), ctx)
    assert (P["n_s"], P["w_s"], P["sample_bits"], P["pred_payload"], P["plan"]) == (4, 2, 7, [40, 4, 12], oracle.FIXEDLEN)
    # one more sampled element of zigzag 0: bits 8, ceil(8 * 10 / 5) = 16 -> same sizes; a minimum gain of 950
    # permil (payload <= 2 bytes) rules both out
    assert oracle.rea_plan_frame(x, EB1, o, oracle.ReaOpts(20, 0), ctx)["pred_payload"] == [40, 4, 12]
    og = oracle.make_opts(chunk_elems=10, alphabet=4, min_gain_permil=950)
    assert oracle.rea_plan_frame(x, EB1, og, oracle.ReaOpts(16, 0), ctx)["plan"] == oracle.RAW
    # an escaped value in the sample (zigzag 8192 >= K - 1): bits (3 + 32) + 1 + 2 + 3 = 41 -> ceil(41 * 10 / 4) = 103
    # bits -> 4 + 4 + 16 = 24 bytes; FIXEDLEN width 14 -> 140 bits -> 20 bytes; totals 64 and 64: tie -> FIXEDLEN
    x2 = x.copy(); x2[0] = _unzig([2 ** 13])[0]
    P2 = oracle.rea_plan_frame(x2, EB1, o, oracle.ReaOpts(16, 0), ctx)
    assert (P2["w_s"], P2["sample_bits"], P2["pred_payload"], P2["plan"]) == (14, 41, [40, 20, 24], oracle.FIXEDLEN)
    # 1000 elements, sample zigzag 0, 0, 0, 2: HUFFMAN 6 bits per 4 symbols -> 1500 bits -> 4 + 8 + 188 = 200 bytes
    # (total 240); FIXEDLEN width 2 -> 2000 bits -> 252 bytes (total 288): HUFFMAN
    o3 = oracle.make_opts(chunk_elems=1000, alphabet=4)
    x3 = _unzig([0, 0, 0, 2] + [1] * 996)
    P3 = oracle.rea_plan_frame(x3, EB1, o3, oracle.ReaOpts(16, 0), ctx)
    assert (P3["sample_bits"], P3["pred_payload"], P3["plan"]) == (6, [4000, 252, 200], oracle.HUFFMAN)
    # the scaling from sample to frame rounds up: 23 elements, 5 sampled (zigzag 0, 0, 0, 1, 1: 7 bits) ->
    # 7 * 23 / 5 = 32.2 -> 33 bits -> two words (rounding down would fit one)
    o4 = oracle.make_opts(chunk_elems=23, alphabet=4)
    x4 = _unzig([0, 0, 0, 1, 1] + [0] * 18)
    P4 = oracle.rea_plan_frame(x4, EB1, o4, oracle.ReaOpts(20, 0), ctx)
    assert (P4["n_s"], P4["sample_bits"], P4["pred_payload"][2]) == (5, 7, 4 + 4 + 8)


@pytest.mark.parametrize("seed", range(12))
def test_plan_equals_exhaustive_minimum_when_the_sample_is_the_frame(seed):
    """With the whole frame inside the sample window the predictions are exact, so Algorithm 1 must commit the
    smallest of the three realized frames (ties to the lower codec id), and the realized payloads must equal the
    predictions."""
    rng = np.random.default_rng(100 + seed)
    nf = int(rng.choice([1, 7, 255, 256, 257, 1000, 4096, 16384]))
    K = int(rng.choice([4, 64, 256, 1024]))
    kind = seed % 4
    if kind == 0:
        x = rng.laplace(0, 1e-3, nf)
    elif kind == 1:
        x = rng.uniform(-1, 1, nf) * rng.choice([1e-3, 1.0])
    elif kind == 2:
        x = np.zeros(nf)
    else:
        x = rng.laplace(0, 1e-3, nf); x[rng.integers(0, nf)] = 0.3
    x = x.astype(np.float32)
    eb = 1e-4
    o = oracle.make_opts(chunk_elems=max(nf, 16), alphabet=K)
    ctx = oracle.context_build(rng.laplace(0, 1e-3, 4000).astype(np.float32), eb, o)
    P = oracle.rea_plan_frame(x, eb, o, None, ctx)
    assert P["n_s"] == nf
    totals = {}
    for c in (0, 1, 2):
        oc = oracle.make_opts(chunk_elems=max(nf, 16), alphabet=K, force_codec=c)
        s, res, rc, _ = oracle.compress_rea(x, eb, oc, None, ctx)
        assert rc == 0
        off, codec, payload, total = _frames(s)[0]
        if codec == c:                                  # (a pinned HUFFMAN larger than RAW falls back)
            totals[c] = total
            assert payload == P["pred_payload"][c]
    best = min(totals, key=lambda c: (totals[c], c))
    s, res, rc, plans = oracle.compress_rea(x, eb, o, None, ctx)
    assert rc == 0 and res.n_fallback == 0 and plans[0] == P["plan"] == best == _frames(s)[0][1]
    # the context's Huffman bits can never beat the frame's own optimal code (optimality of Huffman codes)
    q, _ = oracle.quantize(x, eb)
    assert P["sample_bits"] >= oracle.frame_plan(q, o)["huff_bits"]


def test_realized_output_is_validated_and_raw_is_the_fallback():
    eb = EB1
    o = oracle.make_opts(chunk_elems=40000, alphabet=256)
    ctx = oracle.context_build(_unzig(np.arange(4000) % 5), eb, o)
    # FIXEDLEN planned from a narrow sample (width 3), one later value needs 10 bits -> materialisation fails -> RAW
    z = np.arange(40000) % 5
    x = _unzig(z); x[30000] = 700.0
    of = oracle.make_opts(chunk_elems=40000, alphabet=256, force_codec=1)
    s, res, rc, plans = oracle.compress_rea(x, eb, of, None, ctx)
    assert rc == 0 and plans[0] == oracle.FIXEDLEN and (res.n_raw, res.n_fallback) == (1, 1)
    off, codec, payload, total = _frames(s)[0]
    assert codec == oracle.RAW and (s[off + 32:off + 32 + 4 * x.size].view(np.float32) == x).all()
    # the same value inside the sample widens the plan instead (width 11): no fallback
    x2 = _unzig(z); x2[100] = 700.0
    s, res, rc, plans = oracle.compress_rea(x2, eb, of, None, ctx)
    assert (res.n_fixed, res.n_fallback) == (1, 0) and _frames(s)[0][2] == 4 * ((40000 * 11 + 31) // 32)
    # HUFFMAN planned from a sample of zeros (short codes); the rest of the frame escapes (33+ bits per symbol): the
    # realized payload exceeds the payload capacity -> RAW
    x3 = np.zeros(40000, np.float32); x3[1024:] = _unzig(1000 + np.arange(40000 - 1024) % 3000)
    oh = oracle.make_opts(chunk_elems=40000, alphabet=256, force_codec=2)
    s, res, rc, plans = oracle.compress_rea(x3, eb, oh, oracle.ReaOpts(4096, 0), ctx)
    assert plans[0] == oracle.HUFFMAN and (res.n_raw, res.n_fallback) == (1, 1)
    assert (oracle.decompress(s, x3.size, eb)[0] == x3).all()
    # (unpinned, the all-zero sample plans FIXEDLEN of width 0, which fails on the first non-zero value)
    s, res, rc, plans = oracle.compress_rea(x3, eb, o, oracle.ReaOpts(4096, 0), ctx)
    assert plans[0] == oracle.FIXEDLEN and (res.n_raw, res.n_fallback) == (1, 1)
    # an element that cannot be quantized: inside the sample the plan is RAW at once (no fallback counted), after the
    # sample the coded plan fails and falls back
    x4 = _unzig(z); x4[5] = np.nan
    s, res, rc, plans = oracle.compress_rea(x4, eb, o, None, ctx)
    assert plans[0] == oracle.RAW and (res.n_raw, res.n_fallback) == (1, 0)
    x5 = _unzig(z); x5[39999] = np.inf
    s, res, rc, plans = oracle.compress_rea(x5, eb, o, None, ctx)
    assert plans[0] != oracle.RAW and (res.n_raw, res.n_fallback) == (1, 1)
    assert (s[_frames(s)[0][0] + 32:][:4 * x5.size].view(np.uint32) == x5.view(np.uint32)).all()
    # minimum gain is checked again on the realized size: planned from zeros (gain ~ 97 %), realized 4 bits/symbol
    x6 = np.zeros(40000, np.float32); x6[16384:] = _unzig(np.arange(40000 - 16384) % 14)
    og = oracle.make_opts(chunk_elems=40000, alphabet=256, min_gain_permil=900, force_codec=2)
    ctx6 = oracle.context_build(_unzig(np.arange(4000) % 14), eb, og)
    s, res, rc, plans = oracle.compress_rea(x6, eb, og, None, ctx6)
    assert plans[0] == oracle.HUFFMAN and (res.n_raw, res.n_fallback) == (1, 1)
    og2 = oracle.make_opts(chunk_elems=40000, alphabet=256, min_gain_permil=800, force_codec=2)
    s, res, rc, plans = oracle.compress_rea(x6, eb, og2, None, ctx6)
    assert (res.n_huff, res.n_fallback) == (1, 0)                 # about 3 bits per symbol realized: gain ~ 900 permil


def test_gates():
    eb = 1e-4
    x = W.gradient_like(40000, seed=5)
    o = oracle.make_opts(chunk_elems=20000)
    ctx = oracle.context_build(x[:5000], eb, o)
    assert oracle.compress_rea(x, eb, o, None, ctx)[3].tolist() == [2, 2]
    # Huffman size threshold, missing / foreign context: FIXEDLEN is what is left
    assert oracle.compress_rea(x, eb, oracle.make_opts(chunk_elems=20000, huff_min_bytes=80001), None, ctx)[3].tolist() == [1, 1]
    assert oracle.compress_rea(x, eb, o, None, None)[3].tolist() == [1, 1]
    ctx1024 = oracle.context_build(x[:5000], eb, oracle.make_opts(alphabet=1024))
    assert oracle.compress_rea(x, eb, o, None, ctx1024)[3].tolist() == [1, 1]
    bad = oracle.Context(); assert oracle.compress_rea(x, eb, o, None, bad)[3].tolist() == [1, 1]
    # small-batch fast path: RAW without profiling
    P = oracle.rea_plan_frame(x[:20000], eb, o, oracle.ReaOpts(0, 80001), ctx)
    assert (P["plan"], P["n_s"]) == (oracle.RAW, 0)
    assert oracle.compress_rea(x, eb, o, oracle.ReaOpts(0, 80001), ctx)[1].n_raw == 2
    # the sample window is the prefix: what lies behind it does not change the plan, the window itself does
    xa = x[:20000].copy(); xb = xa.copy(); xb[16384:] = xa[16384:][::-1]
    Pa, Pb = (oracle.rea_plan_frame(v, eb, o, None, ctx) for v in (xa, xb))
    assert Pa == Pb and Pa["n_s"] == 16384
    xc = xa.copy(); xc[:100] = 0.5
    assert oracle.rea_plan_frame(xc, eb, o, None, ctx)["sample_bits"] != Pa["sample_bits"]
    assert oracle.rea_plan_frame(xa, eb, o, oracle.ReaOpts(4096, 0), ctx)["n_s"] == 1024


def test_slotted_stream_layout_and_unchanged_decoder():
    x = W.gradient_like(3 * 20000 + 777, seed=6)
    x[25000] = 0.9                                               # an outlier behind frame 1's sample
    eb = W.abs_bound_from_rel(x, 1e-4)
    o = oracle.make_opts(chunk_elems=20000)
    ctx = oracle.context_build(x[:16384], eb, o)
    s, res, rc, plans = oracle.compress_rea(x, eb, o, None, ctx)
    assert rc == 0 and res.status == 0 and res.n_frames == 4
    base, slot = 64 + 32, (32 + 4 * 20000 + 15) // 16 * 16
    fr = _frames(s)
    assert [f[0] for f in fr] == [base + k * slot for k in range(4)]
    assert res.span_bytes == fr[-1][0] + fr[-1][3] == s.size == int(s[40:48].view(np.uint64)[0])
    assert res.wire_bytes == base + sum(f[3] for f in fr)
    for (off, codec, payload, total), nxt in zip(fr, [f[0] for f in fr[1:]] + [s.size]):
        assert not s[off + 32 + payload:nxt].any()               # padding and the unused part of the slot
    y, dres, drc = oracle.decompress(s, x.size, eb)
    assert drc == 0 and (np.abs(y.astype(np.float64) - x) <= eb).all()
    q, qok = oracle.quantize(x, eb)
    qd, rb, kinds, _, _ = oracle.decode_codes(s, x.size, eb)
    assert kinds.tolist() == [0, 0, 0, 0] and (qd == q).all()
    # frames are never larger than their slot, and the capacity must hold every slot
    cap = oracle.compress_bound(x.size, o)
    assert oracle.compress_rea(x, eb, o, None, ctx, cap=cap)[2] == 0
    s2, res2, rc2, _ = oracle.compress_rea(x, eb, o, None, ctx, cap=cap - 16)
    assert rc2 == oracle.ERR_CAPACITY and res2.span_bytes == 0
    # the result can be reduced like any other stream
    s_exact = oracle.compress(x, eb, o)[0]
    r1 = oracle.reduce_frames(s, s_exact, x.size, eb, o)[0]
    r2 = oracle.reduce_frames(s_exact, s_exact, x.size, eb, o)[0]
    assert r1.tobytes() == r2.tobytes()


def test_against_the_exact_selector_on_gradient_like_data():
    """Per frame the sampled path can only lose to the exact selector (which codes with the frame's own optimal
    code); on stationary data with a context from the first frame the loss is small."""
    x = W.gradient_like(1 << 20, seed=2)
    eb = W.abs_bound_from_rel(x, 1e-4)
    o = oracle.make_opts(chunk_elems=65536)
    ctx = oracle.context_build(x[:65536], eb, o)
    s, res, rc, plans = oracle.compress_rea(x, eb, o, None, ctx)
    e = oracle.compress(x, eb, o)[0]
    fr_r, fr_e = _frames(s), _frames(e)
    assert all(a[3] >= b[3] - 256 for a, b in zip(fr_r, fr_e))    # (the exact frame may carry a shorter length table)
    assert [a[1] for a in fr_r] == [b[1] for b in fr_e]           # same decisions here
    assert res.wire_bytes <= 1.01 * e.size and res.n_fallback == 0


# ------------------------------------------------------------------------------------------------
# Eq. 1 with a transport hint: break-even points in closed form, the limits, and the no-hint case
# ------------------------------------------------------------------------------------------------

def _pad16(v):
    return (v + 15) // 16 * 16


def _model(link=0, fa=0, fp=0, ha=0, hp=0, sample_bytes=0):
    return oracle.ReaOpts(sample_bytes, 0, link, fa, fp, ha, hp, 0)


def test_raw_against_fixedlen_flips_exactly_at_the_break_even_bandwidth():
    """Without a context only RAW and FIXEDLEN compete.  Eq. 1 puts the break-even where the transfer time saved equals
    the codec's exposed time: link_ps * (total_RAW - total_FIXED) = 1000 * alpha_ns + codec_ps * rawBytes.  At that
    point (if it is an integer) and on every faster link RAW is planned, one picosecond per byte slower FIXEDLEN."""
    nf = 50000
    rng = np.random.default_rng(3)
    x = rng.integers(-100, 101, nf).astype(np.float32)                  # zigzag up to 200: w = 8
    o = oracle.make_opts(chunk_elems=nf)
    rawb = 4 * nf
    tot_raw, tot_fix = _pad16(32 + rawb), _pad16(32 + 4 * ((nf * 8 + 31) // 32))
    assert oracle.rea_plan_frame(x, EB1, o, _model(), None)["pred_payload"][1] == tot_fix - 32
    for fa, fp in ((0, 7), (5000, 0), (1234, 3), (0, 1), (4000000, 4000)):
        cost = 1000 * fa + fp * rawb
        be = cost // (tot_raw - tot_fix)                                # largest link_ps at which RAW is still not worse
        if be >= 1:
            assert oracle.rea_plan_frame(x, EB1, o, _model(be, fa, fp), None)["plan"] == oracle.RAW, (fa, fp)
        assert oracle.rea_plan_frame(x, EB1, o, _model(be + 1, fa, fp), None)["plan"] == oracle.FIXEDLEN, (fa, fp)
        if cost % (tot_raw - tot_fix) == 0 and be >= 1:                  # exact tie: the cheaper codec (lower id)
            assert oracle.rea_plan_frame(x, EB1, o, _model(be, fa, fp), None)["plan"] == oracle.RAW
    # an exact tie on purpose: 3 ps per raw byte cost 600000 ps, four times the 150000 bytes saved -> tie at 4 ps/byte
    assert (tot_raw - tot_fix, rawb) == (150000, 200000)
    assert oracle.rea_plan_frame(x, EB1, o, _model(4, 0, 3), None)["plan"] == oracle.RAW
    assert oracle.rea_plan_frame(x, EB1, o, _model(5, 0, 3), None)["plan"] == oracle.FIXEDLEN


def test_huffman_must_amortize_its_extra_codec_cost_over_fixedlen():
    """With a context all three compete.  On a slow link with free codecs the smallest frame wins (HUFFMAN here); as
    HUFFMAN's exposed time per byte grows, FIXEDLEN takes over exactly where
    link * (total_FIXED - total_HUFF) = (huff_ps - fixed_ps) * rawBytes + 1000 * (huff_alpha - fixed_alpha)."""
    nf = 60000
    x = W.gradient_like(nf, seed=6)
    eb = 1e-4
    o = oracle.make_opts(chunk_elems=nf)
    ctx = oracle.context_build(x[:20000], eb, o)
    P = oracle.rea_plan_frame(x, eb, o, _model(), ctx)
    assert P["plan"] == oracle.HUFFMAN
    rawb = 4 * nf
    tot = [_pad16(32 + p) for p in P["pred_payload"]]
    assert tot[2] < tot[1] < tot[0]
    link, fp, fa, ha = 400, 2, 100, 700                                 # 2.5 GB/s: the transfer dominates
    saved = link * (tot[1] - tot[2]) - 1000 * (ha - fa)
    hp_be = fp + saved // rawb                                          # largest huff_ps with cost_H <= cost_F ...
    # ... cost_H < cost_F  <=>  (hp - fp) * rawb < saved
    hp_last = fp + (saved - 1) // rawb
    assert oracle.rea_plan_frame(x, eb, o, _model(link, fa, fp, ha, hp_last), ctx)["plan"] == oracle.HUFFMAN
    assert oracle.rea_plan_frame(x, eb, o, _model(link, fa, fp, ha, hp_last + 1), ctx)["plan"] == oracle.FIXEDLEN
    assert hp_be in (hp_last, hp_last + 1)
    # and on a link so fast that neither codec pays for itself, RAW: the optimal high-bandwidth decision
    assert oracle.rea_plan_frame(x, eb, o, _model(1, 0, 5, 0, 5), ctx)["plan"] == oracle.RAW
    # the gates still apply: a pinned codec ignores the model, T_huff and the minimum gain are checked before the cost
    assert oracle.rea_plan_frame(x, eb, oracle.make_opts(chunk_elems=nf, force_codec=2), _model(1, 0, 5, 0, 5), ctx)["plan"] == oracle.HUFFMAN
    assert oracle.rea_plan_frame(x, eb, oracle.make_opts(chunk_elems=nf, huff_min_bytes=rawb + 1), _model(link), ctx)["plan"] == oracle.FIXEDLEN


def test_no_hint_means_size_only_and_free_codecs_on_any_link_too():
    rng = np.random.default_rng(8)
    nf = 30000
    o = oracle.make_opts(chunk_elems=nf)
    for seed in range(6):
        x = W.gradient_like(nf, seed=20 + seed) if seed % 2 else W.sweep_payload("uniform", nf, 30 + seed)
        eb = float(10.0 ** rng.uniform(-5, -3))
        ctx = oracle.context_build(x[:8000], eb, o)
        base = oracle.rea_plan_frame(x, eb, o, _model(), ctx)
        # link = 0: the other numbers are not looked at
        junk = _model(0, *[int(v) for v in rng.integers(0, 2 ** 31, 4)])
        assert oracle.rea_plan_frame(x, eb, o, junk, ctx) == base
        # codecs that cost nothing: cost = link * total, the same order as the sizes, whatever the link
        for link in (1, 37, 4000, 2 ** 32 - 1):
            assert oracle.rea_plan_frame(x, eb, o, _model(link), ctx)["plan"] == base["plan"]


def test_whole_message_under_a_transport_hint():
    n = 200000
    x = W.gradient_like(n, seed=9)
    eb = 1e-4
    o = oracle.make_opts(chunk_elems=32768)
    ctx = oracle.context_build(x[:16384], eb, o)
    plain, pres, rc0, plans0 = oracle.compress_rea(x, eb, o, _model(), ctx)
    # fast link: every frame is planned RAW (no fallback involved), the message comes back bit for bit
    fast, fres, rc1, plans1 = oracle.compress_rea(x, eb, o, _model(1, 0, 5, 0, 5), ctx)
    assert rc0 == 0 and rc1 == 0 and (plans1 == oracle.RAW).all() and fres.n_raw == fres.n_frames and fres.n_fallback == 0
    y, _, drc = oracle.decompress(fast, n, eb)
    assert drc == 0 and (y.view(np.uint32) == x.view(np.uint32)).all()
    # slow link, free codecs: the very same stream as without a hint
    slow, sres, rc2, plans2 = oracle.compress_rea(x, eb, o, _model(5000), ctx)
    assert rc2 == 0 and (plans2 == plans0).all() and slow.size == plain.size and (slow == plain).all()
    # a reserved field that is not zero is refused
    bad = oracle.ReaOpts(0, 0, 0, 0, 0, 0, 0, 1)
    assert oracle.compress_rea(x, eb, o, bad, ctx)[2] == oracle.ERR_INVALID
    with pytest.raises(ValueError):
        oracle.rea_plan_frame(x[:1000], eb, o, bad, ctx)


# ------------------------------------------------------------------------------------------------
# the ring step with the sampled arbitration on the way out
# ------------------------------------------------------------------------------------------------

def _frame_bytes(stream, k):
    off = int(stream[64 + 8 * k:64 + 8 * k + 8].view(np.uint64)[0])
    payload = int(stream[off + 12:off + 16].view(np.uint32)[0])
    return stream[off:off + 32 + payload]


def test_ring_step_frames_are_the_sampled_frames_of_the_summed_codes():
    """With step = 1 the integer sums of the ring step are themselves fp32 values that quantize to exactly those sums,
    so nzo_reduce_local_rea(in, x) must write, frame for frame and byte for byte, what the (separately pinned)
    nzo_compress_rea writes for the message a + x: same plans, same realized frames, same fallbacks, same counters."""
    rng = np.random.default_rng(41)
    nf, nfr = 20000, 6
    n = nf * nfr - 777
    za = rng.integers(0, 40, n)
    zx = rng.integers(0, 40, n)
    za[2 * nf:3 * nf] = rng.integers(0, 30000, nf)            # frame 2: wide codes -> FIXEDLEN or RAW territory
    zx[3 * nf + 9000] = 20000                                 # frame 3: one wide value behind the sample -> fallback for FIXEDLEN
    za[4 * nf:5 * nf] = 0; zx[4 * nf:5 * nf] = 0              # frame 4: all zero
    a, x = _unzig(za), _unzig(zx)
    assert np.abs(a + x).max() <= 32767
    for kw, rop in ((dict(), None), (dict(force_codec=1), None), (dict(force_codec=2), None), (dict(min_gain_permil=600), None),
                    (dict(), oracle.ReaOpts(4096, 0, 0, 0, 0, 0, 0, 0)), (dict(), oracle.ReaOpts(0, 0, 40, 100, 2, 700, 6, 0))):
        o = oracle.make_opts(chunk_elems=nf, **kw)
        ctx = oracle.context_build(_unzig(rng.integers(0, 60, 30000)), EB1, oracle.make_opts(chunk_elems=nf))
        sa, _, rc = oracle.compress(a, EB1, oracle.make_opts(chunk_elems=nf))
        out, res, rc2, plans = oracle.reduce_local_rea(sa, x, EB1, o, rop, ctx)
        ref, rres, rc3, rplans = oracle.compress_rea(a + x, EB1, o, rop, ctx)
        assert rc == 0 and rc2 == 0 and rc3 == 0
        assert res.as_dict() == rres.as_dict() and (plans == rplans).all(), (kw, res.as_dict(), rres.as_dict())
        for k in range(nfr):
            assert np.array_equal(_frame_bytes(out, k), _frame_bytes(ref, k)), (kw, k)
    assert res.n_frames == nfr


def test_ring_step_codes_raw_rules_and_fallback_values():
    n = 70001
    kw = dict(chunk_elems=20000)
    o = oracle.make_opts(**kw)
    eb = 1e-4
    a, x = W.gradient_like(n, seed=51), W.gradient_like(n, seed=52)
    a[25000] = np.inf                                         # incoming frame 1 RAW
    x[45000] = np.nan                                         # local frame 2 cannot be quantized
    ctx = oracle.context_build(W.gradient_like(30000, seed=53), eb, o)
    sa, _, _ = oracle.compress(a, eb, o)
    out, res, rc, plans = oracle.reduce_local_rea(sa, x, eb, o, None, ctx)
    exact, eres, erc = oracle.reduce_local(sa, x, eb, o)
    assert rc == 0 and erc == 0 and res.n_raw == 2 and res.n_fallback == 0 and list(plans[1:3]) == [0, 0]
    # coded frames carry the exact integer sums; frames without integer sums are the exact path's RAW frames
    q, rb, kinds, _, drc = oracle.decode_codes(out, n, eb)
    qe, rbe, kindse, _, _ = oracle.decode_codes(exact, n, eb)
    assert drc == 0 and (kinds == kindse).all() and (q == qe).all() and (rb == rbe).all()
    qa, _ = oracle.quantize(np.where(np.isfinite(a), a, 0), eb)
    qx, _ = oracle.quantize(np.where(np.isfinite(x), x, 0), eb)
    coded = np.repeat(kinds == 0, 20000)[:n]
    assert (q[coded] == (qa + qx)[coded]).all()
    # the exact selector never loses to the sampled one, frame by frame
    for k in range(4):
        assert _frame_bytes(out, k).size >= _frame_bytes(exact, k).size
    # a coded frame whose realized output is rejected holds the sums of the dequantized operands
    om = oracle.make_opts(min_gain_permil=990, force_codec=2, **kw)
    out2, res2, rc2, plans2 = oracle.reduce_local_rea(sa, x, eb, om, None, ctx)
    assert rc2 == 0 and res2.n_fallback == 2 and res2.n_raw == 4
    y, _, _ = oracle.decompress(out2, n, eb)
    st = oracle.step_constants(eb)[0]
    want = (qa[:20000].astype(np.float32) * st) + (qx[:20000].astype(np.float32) * st)
    assert (y[:20000].view(np.uint32) == want.astype(np.float32).view(np.uint32)).all()
    # refusals
    assert oracle.reduce_local_rea(sa, x, 2e-4, o, None, ctx)[2] == oracle.ERR_MISMATCH
    assert oracle.reduce_local_rea(sa, x, eb, oracle.make_opts(predictor=1, **kw), None, ctx)[2] == oracle.ERR_INVALID
    assert oracle.reduce_local_rea(sa, x, eb, o, oracle.ReaOpts(0, 0, 0, 0, 0, 0, 0, 7), ctx)[2] == oracle.ERR_INVALID
    assert oracle.reduce_local_rea(sa, x, eb, o, None, ctx, cap=1000)[2] == oracle.ERR_CAPACITY
