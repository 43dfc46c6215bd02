"""GPU parity of the sampled runtime entropy arbitration (nz_context_build, nz_compress_rea) against the oracle:
context code lengths, per-frame plan outcome, every byte of every frame, offsets table, stream header and result
record; the slotted stream through the unchanged decoder and the fused reduce."""
import numpy as np
import pytest

import oracle
from paper_2605_12396_amd import workloads as W

pytestmark = pytest.mark.gpu
EB1 = float(np.float32(32.0 / 63.0))          # step = 1 exactly: x = q


@pytest.fixture(scope="module")
def nz(gpu_device):
    from paper_2605_12396_amd import binding
    binding.lib()
    return binding


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def _unzig(z):
    z = np.asarray(z, np.int64)
    return ((z >> 1) ^ -(z & 1)).astype(np.float32)


def gpu_context(nz, cal, eb, g):
    import torch
    ctx = torch.zeros(nz.nz_context_bytes(), dtype=torch.uint8, device="cuda:0")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda:0")
    assert nz.nz_context_build(_dev(cal), cal.size, eb, g, ctx, ws, 4096) == 0
    return ctx


def gpu_rea(nz, x, eb, g, ropts, ctx, cap=None):
    import torch
    n = x.size
    bound = nz.nz_compress_bound(n, nz.make_opts(chunk_elems=g.chunk_elems, alphabet=g.alphabet))
    cap = bound if cap is None else cap
    out = torch.full((max(bound, 16),), 0xAB, dtype=torch.uint8, device="cuda:0")
    res = torch.zeros(nz.REA_RESULT_BYTES + 8, dtype=torch.uint8, device="cuda:0")
    wsb = nz.nz_rea_workspace_bytes(n, g)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda:0")
    rc = nz.nz_compress_rea(_dev(x), n, eb, ctx, out, cap, res, g, ropts, ws, wsb)
    r = nz.read_rea_result(res)
    return rc, r, out


def _frames(stream):
    nfr = int(stream[20:24].view(np.uint32)[0])
    offs = stream[64:64 + 8 * nfr].view(np.uint64).astype(np.int64)
    out = []
    for off in offs:
        h = stream[off:off + 32].view(np.uint32)
        out.append((int(off), int(h[1]), int(h[3]), (32 + int(h[3]) + 15) // 16 * 16))
    return out


def check_rea(nz, x, eb, cal=None, ropts=None, with_ctx=True, **kw):
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    ro_g = nz.ReaOpts(*ropts) if ropts else None
    ro_o = oracle.ReaOpts(*ropts) if ropts else None
    cal = x[:min(x.size, 65536)] if cal is None else cal
    octx = oracle.context_build(cal, eb, o) if with_ctx else None
    gctx = gpu_context(nz, cal, eb, g) if with_ctx else None
    if with_ctx:
        K = o.alphabet or 256
        got_len = gctx[16:16 + 1024].cpu().numpy()
        assert (got_len[:K] == np.array(octx.len[:K])).all() and not got_len[K:].any()
    ref, ores, orc, plans = oracle.compress_rea(x, eb, o, ro_o, octx)
    rc, r, out = gpu_rea(nz, x, eb, g, ro_g, gctx)
    assert rc == 0 and orc == 0 and r == ores.as_dict(), (r, ores.as_dict())
    got = out[:r["span_bytes"]].cpu().numpy()
    base = 64 + (8 * ores.n_frames + 15) // 16 * 16
    assert (got[:base] == ref[:base]).all()                       # stream header and offsets table
    for off, codec, payload, total in _frames(ref):
        d = np.nonzero(got[off:off + total] != ref[off:off + total])[0]
        assert d.size == 0, "frame at %d (codec %d): first differing byte %d" % (off, codec, int(d[0]))
    return ref, ores, out, r, plans


def _cases():
    rng = np.random.default_rng(7)
    x = W.gradient_like(1 << 20, seed=2)
    yield "c2_like_1MBframes", x, W.abs_bound_from_rel(x, 1e-4), dict(chunk_elems=262144), None
    yield "c2_like_K1024", x[:300000], W.abs_bound_from_rel(x, 1e-4), dict(chunk_elems=100000, alphabet=1024), None
    yield "c1_smooth_64KBframes", W.smooth_field((64, 64, 64), seed=1), 1e-4, dict(chunk_elems=16384), None
    yield "ragged_tail", W.gradient_like(70001, seed=4), 1e-4, dict(chunk_elems=20000), None
    yield "chunk_not_multiple_of_4", W.gradient_like(30011, seed=5), 1e-4, dict(chunk_elems=10003), None
    yield "n1", np.array([0.123], np.float32), 1e-3, dict(), None
    yield "n_tiny", W.gradient_like(37, seed=6), 1e-4, dict(chunk_elems=16), None
    yield "piece_tails", W.gradient_like(3 * 4096 + 5, seed=9), 1e-4, dict(chunk_elems=4096 + 1), None
    yield "max_chunk", W.gradient_like((1 << 20) + 5000, seed=7), 3e-4, dict(chunk_elems=1 << 20), None
    yield "uniform_fixedlen", W.sweep_payload("uniform", 200000, 50), 1e-4, dict(chunk_elems=65536), None
    yield "all_zero", np.zeros(50000, np.float32), 1e-4, dict(chunk_elems=16384), None
    yield "escape_heavy_K16", (rng.laplace(0, 3e-3, 100000)).astype(np.float32), 1e-4, dict(chunk_elems=32768, alphabet=16), None
    yield "K2", (rng.laplace(0, 1e-4, 60000)).astype(np.float32), 1e-4, dict(chunk_elems=32768, alphabet=2), None
    yield "small_sample", W.gradient_like(200000, seed=8), 1e-4, dict(chunk_elems=65536), (4096, 0)
    yield "sample_whole_frame", W.gradient_like(200000, seed=8), 1e-4, dict(chunk_elems=65536), (1 << 20, 0)
    yield "small_batch_raw", W.gradient_like(50000, seed=8), 1e-4, dict(chunk_elems=16384), (0, 65537)
    y = W.gradient_like(100000, seed=8)
    y[[5, 40000, 99999]] = [np.nan, np.inf, -1e30]              # frame 0: in the sample; frames 2, 6: behind it
    yield "nan_inf_frames", y, 1e-4, dict(chunk_elems=16384), (16384, 0)
    z = W.gradient_like(200000, seed=10); z[[70000, 150000]] = [0.7, -0.9]
    yield "late_outliers_fixed_fallback", z, 1e-4, dict(chunk_elems=65536, force_codec=1), None
    yield "pinned_raw", W.gradient_like(50000, seed=11), 1e-4, dict(chunk_elems=16384, force_codec=0), None
    yield "pinned_huffman_uniform", W.sweep_payload("uniform", 100000, 52), 1e-4, dict(chunk_elems=32768, force_codec=2), None
    yield "gates", W.gradient_like(100000, seed=12), 1e-4, dict(chunk_elems=25000, huff_min_bytes=100001, min_gain_permil=300), None


@pytest.mark.parametrize("name,x,eb,kw,ropts", list(_cases()), ids=[c[0] for c in _cases()])
def test_rea_frames_match_oracle_and_decode(nz, name, x, eb, kw, ropts):
    import torch
    ref, ores, out, r, plans = check_rea(nz, x, eb, ropts=ropts, **kw)
    # the slotted stream through the unchanged GPU decoder: the oracle's values, the bound
    g = nz.make_opts(**{k: v for k, v in kw.items() if k in ("chunk_elems", "alphabet")})
    sess = nz.Session(x.size, g, "cuda:0")
    y = torch.full((x.size,), 7.0, dtype=torch.float32, device="cuda:0")
    rc, y = sess.decompress(out, r["span_bytes"], x.size, eb, out=y)
    rr = sess.result()
    yo, dres, drc = oracle.decompress(ref, x.size, eb)
    assert rc == 0 and drc == 0 and rr["status"] == 0 and (rr["n_raw"], rr["n_fixed"], rr["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    y = y.cpu().numpy()
    assert (y.view(np.uint32) == yo.view(np.uint32)).all()
    fin = np.isfinite(x)
    assert (np.abs(y[fin].astype(np.float64) - x[fin]) <= np.float32(eb)).all()


def test_rea_without_context_and_foreign_context(nz):
    x = W.gradient_like(100000, seed=13)
    ref, ores, *_ = check_rea(nz, x, 1e-4, with_ctx=False, chunk_elems=32768)
    assert ores.n_huff == 0 and ores.n_fixed == 4
    # a context built for another alphabet is not valid for this one
    g, o = nz.make_opts(chunk_elems=32768), oracle.make_opts(chunk_elems=32768)
    gctx = gpu_context(nz, x[:5000], 1e-4, nz.make_opts(alphabet=1024))
    rc, r, out = gpu_rea(nz, x, 1e-4, g, None, gctx)
    assert rc == 0 and (r["n_huff"], r["n_fixed"]) == (0, 4)
    # a context from different data still gives valid (if larger) frames, identical to the oracle's
    check_rea(nz, x, 1e-4, cal=W.sweep_payload("uniform", 30000, 3) * 0.01, chunk_elems=32768)


def test_rea_realized_size_fallbacks(nz):
    # HUFFMAN planned from a sample of zeros, the rest escapes: realized payload larger than RAW -> RAW; the pieces go
    # through the encoder's pass-by-pass path (more than 16 bits per symbol)
    o = dict(chunk_elems=40000, alphabet=256, force_codec=2)
    cal = _unzig(np.arange(4000) % 5)
    x3 = np.zeros(40000, np.float32); x3[1024:] = _unzig(1000 + np.arange(40000 - 1024) % 3000)
    ref, ores, *_ = check_rea(nz, x3, EB1, cal=cal, ropts=(4096, 0), **o)
    assert (ores.n_raw, ores.n_fallback) == (1, 1)
    # half of the symbols escape (about 20 bits per symbol on average): pass-by-pass path, accepted
    z = np.arange(120000) % 5
    z[::2] = 1000 + (np.arange(60000) % 2000)
    ref, ores, *_ = check_rea(nz, _unzig(z), EB1, cal=cal, chunk_elems=50000, alphabet=256, force_codec=2)
    assert (ores.n_huff, ores.n_fallback) == (3, 0)
    # minimum gain on the realized size
    x6 = np.zeros(40000, np.float32); x6[16384:] = _unzig(np.arange(40000 - 16384) % 14)
    cal6 = _unzig(np.arange(4000) % 14)
    ref, ores, *_ = check_rea(nz, x6, EB1, cal=cal6, chunk_elems=40000, min_gain_permil=900, force_codec=2)
    assert (ores.n_raw, ores.n_fallback) == (1, 1)
    ref, ores, *_ = check_rea(nz, x6, EB1, cal=cal6, chunk_elems=40000, min_gain_permil=800, force_codec=2)
    assert (ores.n_huff, ores.n_fallback) == (1, 0)


def test_rea_deepest_context_codes(nz):
    """A context whose (count + 1) weights form a Fibonacci-like chain has 27-bit codes; a frame that starts with its
    rarest symbols side by side puts more than 64 bits into one thread's four symbols."""
    chain = [6, 10, 16, 26, 42, 68, 110, 178, 288, 466, 754, 1220, 1974, 3194, 5168, 8362, 13530, 21892, 35422, 57314,
             92736, 150050, 242786]                               # weights of zigzag codes 0..22; the other symbols weigh 1
    cal = _unzig(np.concatenate([np.full(c - 1, i) for i, c in enumerate(chain)]))
    assert cal.size <= 1 << 20
    octx = oracle.context_build(cal, EB1, oracle.make_opts(alphabet=32))
    assert max(octx.len[:32]) == 27
    rng = np.random.default_rng(8)
    z = rng.integers(0, 23, 150000)
    z[:64] = np.arange(64) % 4                                    # the rarest symbols (24+ bits each) side by side
    z[4096 * 3:4096 * 3 + 2000] = np.arange(2000) % 3
    ref, ores, *_ = check_rea(nz, _unzig(z), EB1, cal=cal, chunk_elems=65536, alphabet=32, force_codec=2)
    assert ores.n_huff == 3


def test_rea_capacity_and_arguments(nz):
    import torch
    x = W.gradient_like(100000, seed=14)
    g = nz.make_opts(chunk_elems=16384)
    gctx = gpu_context(nz, x[:10000], 1e-4, g)
    bound = nz.nz_compress_bound(x.size, g)
    rc, r, out = gpu_rea(nz, x, 1e-4, g, None, gctx, cap=bound - 16)
    assert rc == nz.ERR_CAPACITY and r["status"] == nz.ERR_CAPACITY and r["span_bytes"] == 0
    assert bool((out == 0xAB).all())                              # nothing written
    rc, r, out = gpu_rea(nz, x, 1e-4, g, None, gctx, cap=bound)
    assert rc == 0 and r["status"] == 0
    res = torch.zeros(48, dtype=torch.uint8, device="cuda:0")
    ws = torch.empty(nz.nz_rea_workspace_bytes(x.size, g), dtype=torch.uint8, device="cuda:0")
    dx = _dev(x)
    assert nz.nz_compress_rea(dx, 0, 1e-4, gctx, out, bound, res, g, None, ws, ws.numel()) == nz.ERR_INVALID
    assert nz.nz_compress_rea(dx, x.size, 0.0, gctx, out, bound, res, g, None, ws, ws.numel()) == nz.ERR_INVALID
    assert nz.nz_compress_rea(dx, x.size, 1e-4, gctx, out, bound, res, g, None, ws, 16) == nz.ERR_INVALID
    assert nz.nz_compress_rea(dx, x.size, 1e-4, gctx, out, bound, res, nz.make_opts(seg_syms=64), None, ws, ws.numel()) == nz.ERR_INVALID
    assert nz.nz_context_build(dx, (1 << 20) + 1, 1e-4, g, gctx, ws, ws.numel()) == nz.ERR_INVALID
    torch.cuda.synchronize()


def test_rea_stream_feeds_the_fused_reduce(nz):
    import torch
    n, eb = 300000, 1e-5
    kw = dict(chunk_elems=65536)
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    a, b = W.gradient_like(n, seed=40, outlier_frac=0.0), W.gradient_like(n, seed=41, outlier_frac=0.0)
    ref_a, ores, out_a, r_a, _ = check_rea(nz, a, eb, **kw)
    sb = oracle.compress(b, eb, o)[0]
    red, rres, rrc = oracle.reduce_frames(ref_a, sb, n, eb, o)
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    db = _dev(np.concatenate([sb, np.zeros((-sb.size) % 16, np.uint8)]))
    rc, got = sess.reduce(out_a, r_a["span_bytes"], db, sb.size, n, eb)
    r = sess.result()
    assert rc == 0 and rrc == 0 and r["status"] == 0 and r["bytes"] == rres.bytes
    assert (got[:r["bytes"]].cpu().numpy() == red).all()
    rc, got = sess.reduce_local(out_a, r_a["span_bytes"], _dev(b), n, eb)
    r = sess.result()
    assert rc == 0 and r["status"] == 0 and (got[:r["bytes"]].cpu().numpy() == red).all()


def test_rea_repeatable_and_c2_full_size(nz):
    """The headline message through the sampled path, in the launch configuration bench.py times: every frame against
    the oracle; and the same call three times gives the same bytes (the look-back order does not matter)."""
    n = 1 << 26
    x = W.gradient_like(n, seed=2)
    eb = float(np.float32(W.abs_bound_from_rel(x, 1e-4)))
    ref, ores, out, r, plans = check_rea(nz, x, eb, chunk_elems=262144)
    assert ores.n_huff == 256 and ores.n_fallback == 0
    g = nz.make_opts(chunk_elems=262144)
    gctx = gpu_context(nz, x[:65536], eb, g)
    first = out[:r["span_bytes"]].clone()
    for _ in range(3):
        rc, r2, out2 = gpu_rea(nz, x, eb, g, None, gctx)
        for off, codec, payload, total in _frames(ref)[::17]:
            assert bool((out2[off:off + total] == first[off:off + total]).all())


@pytest.mark.parametrize("model", [
    (0, 0, 1, 0, 5, 0, 5, 0),                # a link so fast that no codec pays for itself: every frame planned RAW
    (0, 0, 40, 100, 2, 700, 6, 0),           # 25 GB/s, HUFFMAN three times as expensive as FIXEDLEN
    (0, 0, 400, 100, 2, 700, 60, 0),         # 2.5 GB/s, HUFFMAN's exposed time too high: FIXEDLEN or RAW
    (0, 0, 5000, 0, 0, 0, 0, 0),             # slow link, free codecs: the sizes decide
    (4096, 0, 12, 20000, 0, 20000, 0, 0),    # fixed costs only, short sample window
], ids=["fast_link", "mid_link", "huffman_too_slow", "slow_link_free_codecs", "fixed_costs"])
def test_plans_under_a_transport_hint_match_the_oracle(nz, model):
    """Eq. 1 with the caller's transport hint and codec costs: same plans, same frames, same counters as the oracle, on
    a message whose frames differ in compressibility (gradient-like, uniform, smooth, all zero)."""
    n = 6 * 32768 + 1234
    x = np.concatenate([W.gradient_like(2 * 32768, seed=3), W.sweep_payload("uniform", 2 * 32768, 4),
                        W.smooth_field((32, 32, 32), seed=5).reshape(-1), np.zeros(32768 + 1234, np.float32)])
    assert x.size == n
    ref, ores, out, r, plans = check_rea(nz, x, 1e-4, cal=x[:65536], ropts=model, chunk_elems=32768)
    if model[2] == 1:
        assert (plans == oracle.RAW).all() and r["n_raw"] == r["n_frames"] and r["n_fallback"] == 0
    if model[2] == 5000:
        plain = oracle.compress_rea(x, 1e-4, oracle.make_opts(chunk_elems=32768), None,
                                    oracle.context_build(x[:65536], 1e-4, oracle.make_opts(chunk_elems=32768)))[0]
        assert plain.size == ref.size and (plain == ref).all()


def test_reserved_option_field_is_refused(nz):
    import torch
    n = 1000
    g = nz.make_opts(chunk_elems=256)
    x = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    cap = nz.nz_compress_bound(n, g)
    out = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
    res = torch.zeros(48, dtype=torch.uint8, device="cuda:0")
    wsb = nz.nz_rea_workspace_bytes(n, g)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda:0")
    bad = nz.ReaOpts(0, 0, 0, 0, 0, 0, 0, 1)
    assert nz.nz_compress_rea(x, n, 1e-4, None, out, cap, res, g, bad, ws, wsb) == nz.ERR_INVALID
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------------
# the ring step with the sampled arbitration on the way out
# ------------------------------------------------------------------------------------------------

def gpu_reduce_local_rea(nz, a_stream, x, eb, g, ropts, ctx, cap=None):
    import torch
    n = x.size
    bound = nz.nz_compress_bound(n, nz.make_opts(chunk_elems=g.chunk_elems, alphabet=g.alphabet))
    cap = bound if cap is None else cap
    out = torch.full((max(bound, 16),), 0xAB, dtype=torch.uint8, device="cuda:0")
    res = torch.zeros(nz.REA_RESULT_BYTES + 8, dtype=torch.uint8, device="cuda:0")
    wsb = nz.nz_reduce_rea_workspace_bytes(n, g)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda:0")
    da = _dev(np.concatenate([a_stream, np.zeros((-a_stream.size) % 16, np.uint8)]))
    rc = nz.nz_reduce_local_rea(da, a_stream.size, _dev(x), n, eb, ctx, out, cap, res, g, ropts, ws, wsb)
    return rc, nz.read_rea_result(res), out


def check_ring_rea(nz, a, x, eb, ropts=None, with_ctx=True, a_kw=None, **kw):
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    ro_g = nz.ReaOpts(*ropts) if ropts else None
    ro_o = oracle.ReaOpts(*ropts) if ropts else None
    base_kw = dict(chunk_elems=kw.get("chunk_elems", 0), alphabet=kw.get("alphabet", 0))
    sa, _, rc0 = oracle.compress(a, eb, oracle.make_opts(**(a_kw or base_kw)))
    cal = x[:min(x.size, 65536)]
    octx = oracle.context_build(cal, eb, o) if with_ctx else None
    gctx = gpu_context(nz, cal, eb, g) if with_ctx else None
    ref, ores, orc, plans = oracle.reduce_local_rea(sa, x, eb, o, ro_o, octx)
    rc, r, out = gpu_reduce_local_rea(nz, sa, x, eb, g, ro_g, gctx)
    assert rc0 == 0 and rc == 0 and orc == 0 and r == ores.as_dict(), (r, ores.as_dict())
    got = out[:r["span_bytes"]].cpu().numpy()
    base = 64 + (8 * ores.n_frames + 15) // 16 * 16
    assert (got[:base] == ref[:base]).all()
    for off, codec, payload, total in _frames(ref):
        d = np.nonzero(got[off:off + total] != ref[off:off + total])[0]
        assert d.size == 0, "frame at %d (codec %d): first differing byte %d" % (off, codec, int(d[0]))
    return ref, ores, out, r, plans


def _ring_cases():
    n = 300000
    a, x = W.gradient_like(n, seed=71), W.gradient_like(n, seed=72)
    yield "gradient_256KBframes", a, x, 1e-4, None, dict(chunk_elems=65536)
    yield "gradient_1MBframes", W.gradient_like(700000, seed=73), W.gradient_like(700000, seed=74), 1e-4, None, dict(chunk_elems=262144)
    yield "K1024", a, x, 1e-5, None, dict(chunk_elems=100000, alphabet=1024)
    yield "ragged_small_frames", a[:30011], x[:30011], 1e-4, None, dict(chunk_elems=10003)
    yield "tiny", a[:37], x[:37], 1e-4, None, dict(chunk_elems=16)
    yield "uniform_fixedlen", W.sweep_payload("uniform", 200000, 75), W.sweep_payload("uniform", 200000, 76), 1e-4, None, dict(chunk_elems=65536)
    yield "pinned_huffman", a, x, 1e-4, None, dict(chunk_elems=65536, force_codec=2)
    yield "pinned_fixedlen", a, x, 1e-4, None, dict(chunk_elems=65536, force_codec=1)
    yield "pinned_raw", a, x, 1e-4, None, dict(chunk_elems=65536, force_codec=0)
    yield "min_gain_rejects_everything", a, x, 1e-4, None, dict(chunk_elems=65536, min_gain_permil=990)
    yield "short_sample", a, x, 1e-4, (1024, 0, 0, 0, 0, 0, 0, 0), dict(chunk_elems=65536)
    yield "small_batch_fast_path", a, x, 1e-4, (0, 1 << 20, 0, 0, 0, 0, 0, 0), dict(chunk_elems=65536)
    yield "fast_link_all_raw", a, x, 1e-4, (0, 0, 1, 0, 5, 0, 5, 0), dict(chunk_elems=65536)
    yield "mid_link", a, x, 1e-4, (0, 0, 40, 100, 2, 700, 6, 0), dict(chunk_elems=65536)
    a2, x2 = a.copy(), x.copy()
    a2[70000] = np.inf; x2[140000] = np.nan; x2[250000] = 1e30
    yield "frames_without_integer_sums", a2, x2, 1e-4, None, dict(chunk_elems=65536)
    # one value behind the sample (the first 64 KiB of a frame) is wider than anything in it: a FIXEDLEN plan fails when
    # realized, a HUFFMAN plan escapes it
    a3, x3 = a.copy(), x.copy()
    x3[65536 + 30000] = 6.0                                            # 16 bits, wider than anything in the sample
    yield "wide_behind_the_sample", a3, x3, 1e-4, None, dict(chunk_elems=65536)
    yield "wide_behind_the_sample_fixedlen", a3, x3, 1e-4, None, dict(chunk_elems=65536, force_codec=1)


@pytest.mark.parametrize("name,a,x,eb,ropts,kw", list(_ring_cases()), ids=[c[0] for c in _ring_cases()])
def test_ring_step_with_sampled_arbitration_matches_oracle(nz, name, a, x, eb, ropts, kw):
    ref, ores, out, r, plans = check_ring_rea(nz, a, x, eb, ropts=ropts, **kw)
    if name == "fast_link_all_raw":
        assert (plans == oracle.RAW).all() and r["n_fallback"] == 0
    if name == "frames_without_integer_sums":
        assert r["n_raw"] >= 3 and r["n_fallback"] == 0
    if name == "wide_behind_the_sample_fixedlen":
        assert r["n_fallback"] >= 1
    if name == "min_gain_rejects_everything":
        assert r["n_raw"] == r["n_frames"]


def test_ring_step_sampled_without_context_and_errors(nz):
    import torch
    n = 100000
    a, x = W.gradient_like(n, seed=81), W.gradient_like(n, seed=82)
    kw = dict(chunk_elems=32768)
    check_ring_rea(nz, a, x, 1e-4, with_ctx=False, **kw)                 # no context: FIXEDLEN or RAW only
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    sa, _, _ = oracle.compress(a, 1e-4, o)
    # a stream made with another bound, a corrupted frame: status carried over, nothing published
    rc, r, out = gpu_reduce_local_rea(nz, sa, x, 2e-4, g, None, None)
    assert rc == 0 and r["status"] == nz.ERR_MISMATCH and r["span_bytes"] == 0 and r["wire_bytes"] == 0
    bad = sa.copy()
    off = int(bad[64 + 8:64 + 16].view(np.uint64)[0])
    bad[off + 4] ^= 0x40
    rc, r, out = gpu_reduce_local_rea(nz, bad, x, 1e-4, g, None, None)
    assert rc == 0 and r["status"] == nz.ERR_CORRUPT and r["span_bytes"] == 0
    assert oracle.reduce_local_rea(bad, x, 1e-4, o, None, None)[2] == oracle.ERR_CORRUPT
    # capacity one slot short, predictor, reserved field
    bound = nz.nz_compress_bound(n, g)
    rc, r, out = gpu_reduce_local_rea(nz, sa, x, 1e-4, g, None, None, cap=bound - 16)
    assert rc == nz.ERR_CAPACITY and r["status"] == nz.ERR_CAPACITY
    assert gpu_reduce_local_rea(nz, sa, x, 1e-4, nz.make_opts(predictor=1, **kw), None, None)[0] == nz.ERR_INVALID
    assert gpu_reduce_local_rea(nz, sa, x, 1e-4, g, nz.ReaOpts(0, 0, 0, 0, 0, 0, 0, 3), None)[0] == nz.ERR_INVALID
    assert nz.nz_reduce_rea_workspace_bytes(n, nz.make_opts(seg_syms=64)) == 0
    torch.cuda.synchronize()


def test_ring_step_sampled_c2_full_size(nz):
    """The headline geometry (64 Mi elements, 1 MiB frames) through the sampled ring step, in the launch configuration
    bench.py times: every frame against the oracle."""
    n = 1 << 26
    a = W.gradient_like(n, seed=2)
    x = W.gradient_like(n, seed=102)
    eb = float(np.float32(W.abs_bound_from_rel(a, 1e-4)))
    ref, ores, out, r, plans = check_ring_rea(nz, a, x, eb, chunk_elems=262144)
    assert ores.n_huff == 256 and ores.n_fallback == 0
