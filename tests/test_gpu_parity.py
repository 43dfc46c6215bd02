"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: compressed / reduced streams bit-identical (bytes, selector decisions, sizes); decompressed fp32 values
bit-identical (both sides compute fl32(float(q)*step), so the 1-ulp allowance is not needed); |x - xhat| <= eb
checked in float64 as a hard invariant.
"""
import numpy as np
import pytest

import oracle
from paper_2605_12396_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nz(gpu_device):
    from paper_2605_12396_amd import binding
    binding.lib()
    return binding


def _opts_pair(nz, **kw):
    return nz.make_opts(**kw), oracle.make_opts(**kw)


def _to_dev(nz, x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def gpu_compress(nz, x, eb, g_opts, cap=None):
    sess = nz.Session(x.size, g_opts, "cuda:0")
    rc, out = sess.compress(_to_dev(nz, x), eb, cap=cap)
    r = sess.result()
    return rc, r, out[:r["bytes"]].cpu().numpy()


def gpu_decompress(nz, stream, n, eb, g_opts):
    import torch
    sess = nz.Session(n, g_opts, "cuda:0")
    pad = (-stream.size) % 16
    d = _to_dev(nz, np.concatenate([stream, np.zeros(pad, np.uint8)]))
    out = torch.full((n,), 7.0, dtype=torch.float32, device="cuda:0")
    rc, out = sess.decompress(d, stream.size, n, eb, out=out)
    r = sess.result()
    return rc, r, out.cpu().numpy()


def gpu_reduce(nz, a, b, n, eb, g_opts, cap=None):
    sess = nz.Session(n, g_opts, "cuda:0", reduce=True)
    da = _to_dev(nz, np.concatenate([a, np.zeros((-a.size) % 16, np.uint8)]))
    db = _to_dev(nz, np.concatenate([b, np.zeros((-b.size) % 16, np.uint8)]))
    rc, out = sess.reduce(da, a.size, db, b.size, n, eb, cap=cap)
    r = sess.result()
    return rc, r, out[:r["bytes"]].cpu().numpy()


def _first_diff(a, b):
    m = min(a.size, b.size)
    d = np.nonzero(a[:m] != b[:m])[0]
    return int(d[0]) if d.size else (m if a.size != b.size else -1)


def gpu_reduce_local(nz, a, x, eb, g_opts, cap=None):
    n = x.size
    sess = nz.Session(n, g_opts, "cuda:0", reduce=True)
    da = _to_dev(nz, np.concatenate([a, np.zeros((-a.size) % 16, np.uint8)]))
    rc, out = sess.reduce_local(da, a.size, _to_dev(nz, x), n, eb, cap=cap)
    r = sess.result()
    return rc, r, out[:r["bytes"]].cpu().numpy()


def check_compress(nz, x, eb, **kw):
    g, o = _opts_pair(nz, **kw)
    ref, ores, orc = oracle.compress(x, eb, o)
    rc, r, got = gpu_compress(nz, x, eb, g)
    assert rc == 0 and orc == 0 and r["status"] == 0, (rc, orc, r)
    assert (r["n_raw"], r["n_fixed"], r["n_huff"], r["n_frames"]) == (ores.n_raw, ores.n_fixed, ores.n_huff, ores.n_frames)
    assert r["bytes"] == ores.bytes, (r, ores.as_dict())
    assert _first_diff(got, ref) == -1, "first differing byte at %d" % _first_diff(got, ref)
    return ref, ores


def check_decompress(nz, stream, x, eb, **kw):
    g, o = _opts_pair(nz, **kw)
    ref, ores, orc = oracle.decompress(stream, x.size, eb)
    rc, r, got = gpu_decompress(nz, stream, x.size, eb, g)
    assert rc == 0 and orc == 0 and r["status"] == 0, (rc, orc, r)
    assert r["bytes"] == stream.size
    assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    assert (got.view(np.uint32) == ref.view(np.uint32)).all()
    finite = np.isfinite(x)
    err = np.abs(got[finite].astype(np.float64) - x[finite].astype(np.float64))
    assert (err <= np.float32(eb)).all()                     # hard invariant (RAW frames reproduce x exactly)


# ------------------------------------------------------------------------------------------------
# compress + decompress
# ------------------------------------------------------------------------------------------------

def _cases():
    rng = np.random.default_rng(99)
    yield "c1_smooth_64KBframes", W.smooth_field((256, 64, 64), seed=1), 1e-4, dict(chunk_elems=16384)
    x = W.gradient_like(1 << 20, seed=2)
    yield "c2_like_1MBframes", x, W.abs_bound_from_rel(x, 1e-4), dict(chunk_elems=262144)
    yield "c2_like_K1024", x[:300000], W.abs_bound_from_rel(x, 1e-4), dict(chunk_elems=100000, alphabet=1024)
    yield "ragged_tail", W.gradient_like(70001, seed=4), 1e-4, dict(chunk_elems=20000)
    yield "chunk_not_multiple_of_4", W.gradient_like(30011, seed=5), 1e-4, dict(chunk_elems=10003)
    yield "n1", np.array([0.123], np.float32), 1e-3, dict()
    yield "n_tiny", W.gradient_like(37, seed=6), 1e-4, dict(chunk_elems=16)
    yield "max_chunk", W.gradient_like((1 << 20) + 5000, seed=7), 3e-4, dict(chunk_elems=1 << 20)
    yield "uniform_fixedlen", W.sweep_payload("uniform", 200000, 50), 1e-4, dict(chunk_elems=65536)
    yield "sinusoid", W.sweep_payload("sinusoid", 200000, 51), 1e-4, dict(chunk_elems=16384)
    yield "all_zero", np.zeros(50000, np.float32), 1e-4, dict(chunk_elems=16384)
    yield "constant", np.full(50000, 0.777, np.float32), 1e-4, dict(chunk_elems=16384)
    yield "escape_heavy_K16", (rng.laplace(0, 3e-3, 100000)).astype(np.float32), 1e-4, dict(chunk_elems=32768, alphabet=16)
    yield "K2", (rng.laplace(0, 1e-4, 60000)).astype(np.float32), 1e-4, dict(chunk_elems=32768, alphabet=2)
    y = W.gradient_like(100000, seed=8)
    y[[5, 40000, 99999]] = [np.nan, np.inf, -1e30]
    yield "nan_inf_frames_raw", y, 1e-4, dict(chunk_elems=16384)
    z = (rng.uniform(-1, 1, 80000) * 32767 * 1.96875e-3).astype(np.float32)
    yield "codes_up_to_qmax", z, 1e-3, dict(chunk_elems=16384)
    yield "denormals_and_tiny_eb", (rng.standard_normal(40000) * 1e-38).astype(np.float32), 1e-30, dict(chunk_elems=8192)


@pytest.mark.parametrize("name,x,eb,kw", list(_cases()), ids=[c[0] for c in _cases()])
def test_compress_bytes_and_decompress_values_match_oracle(nz, name, x, eb, kw):
    ref, _ = check_compress(nz, x, eb, **kw)
    check_decompress(nz, ref, x, eb, **kw)


@pytest.mark.parametrize("codec", [0, 1, 2])
@pytest.mark.parametrize("kind", ["laplace", "uniform", "sinusoid"])
def test_pinned_codecs(nz, codec, kind):
    x = W.sweep_payload(kind, 150000, 60)
    kw = dict(chunk_elems=40000, force_codec=codec)
    ref, _ = check_compress(nz, x, 1e-4, **kw)
    check_decompress(nz, ref, x, 1e-4, **kw)


def test_selector_gates(nz):
    x = W.gradient_like(200000, seed=12)
    for kw in (dict(chunk_elems=50000, huff_min_bytes=200001), dict(chunk_elems=50000, min_gain_permil=700),
               dict(chunk_elems=50000, min_gain_permil=1000), dict(chunk_elems=50000, huff_min_bytes=4 * 50000)):
        check_compress(nz, x, 1e-4, **kw)


def test_repeatable(nz):
    x = W.gradient_like(500000, seed=13)
    g, _ = _opts_pair(nz, chunk_elems=65536)
    first = gpu_compress(nz, x, 1e-4, g)[2]
    for _ in range(3):
        assert (gpu_compress(nz, x, 1e-4, g)[2] == first).all()


def test_capacity_and_argument_errors(nz):
    import torch
    x = W.gradient_like(100000, seed=14)
    g, o = _opts_pair(nz, chunk_elems=16384)
    ref, ores, _ = oracle.compress(x, 1e-4, o)
    for cap in (int(ores.bytes) - 16, 4096, 64):
        rc, r, _ = gpu_compress(nz, x, 1e-4, g, cap=cap)
        assert r["status"] == nz.ERR_CAPACITY and r["bytes"] == 0
    rc, r, got = gpu_compress(nz, x, 1e-4, g, cap=int(ores.bytes))
    assert rc == 0 and r["status"] == 0 and (got == ref).all()
    sess = nz.Session(x.size, g, "cuda:0")
    dx = _to_dev(nz, x)
    out = sess.new_stream_buffer()
    for eb in (0.0, -1.0, float("nan"), float("inf"), 1e-35):
        assert nz.nz_compress(dx, x.size, eb, out, sess.cap, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_compress(dx, 0, 1e-4, out, sess.cap, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_compress(dx, x.size, 1e-4, out, sess.cap, sess.res, g, sess.ws, 16) == nz.ERR_INVALID
    assert nz.nz_compress(dx[1:], x.size - 1, 1e-4, out, sess.cap, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    bad = nz.make_opts(chunk_elems=16384, seg_syms=128)
    assert nz.nz_compress(dx, x.size, 1e-4, out, sess.cap, sess.res, bad, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    torch.cuda.synchronize()


def test_decompress_rejections(nz):
    x = W.gradient_like(60000, seed=15)
    eb = 1e-4
    g, o = _opts_pair(nz, chunk_elems=16384)
    s, _, _ = oracle.compress(x, eb, o)
    ref, _, _ = oracle.decompress(s, x.size, eb)
    # stream-level
    assert gpu_decompress(nz, s, x.size, 2e-4, g)[1]["status"] == nz.ERR_MISMATCH
    g2 = nz.make_opts(chunk_elems=8192)
    assert gpu_decompress(nz, s, x.size, eb, g2)[1]["status"] == nz.ERR_MISMATCH
    t = s.copy(); t[0] ^= 1
    assert gpu_decompress(nz, t, x.size, eb, g)[1]["status"] == nz.ERR_CORRUPT
    assert gpu_decompress(nz, s[:-16], x.size, eb, g)[1]["status"] == nz.ERR_CORRUPT
    # frame headers: same verdict as the oracle, and the same output everywhere -- a rejected frame is zero-filled
    off = int(s[64 + 8:64 + 16].view(np.uint64)[0])
    for i in range(32):
        t = s.copy(); t[off + i] ^= 0x41
        oref, ores, orc = oracle.decompress(t, x.size, eb)
        rc, r, got = gpu_decompress(nz, t, x.size, eb, g)
        assert r["status"] == orc, (i, r, orc)
        assert (r["n_raw"], r["n_fixed"], r["n_huff"], r["bytes"]) == (ores.n_raw, ores.n_fixed, ores.n_huff, ores.bytes)
        assert (got.view(np.uint32) == oref.view(np.uint32)).all(), i
    # garbage inside payloads: never faults; same verdict and same output as the oracle (a frame found corrupt while
    # decoding is zero-filled as a whole, the others are untouched)
    rng = np.random.default_rng(3)
    n_rejected = 0
    for _ in range(60):
        t = s.copy()
        i = int(rng.integers(off + 32, s.size))
        t[i] ^= int(rng.integers(1, 256))
        oref, ores, orc = oracle.decompress(t, x.size, eb)
        rc, r, got = gpu_decompress(nz, t, x.size, eb, g)
        assert r["status"] == orc, (i, r, orc)
        assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
        assert (got.view(np.uint32) == oref.view(np.uint32)).all(), i
        n_rejected += orc != 0
    assert n_rejected > 10
    # a frame larger than one decode workgroup, broken in its last workgroup's share: the whole frame is cleared
    g3, o3 = _opts_pair(nz, chunk_elems=200000)
    x3 = W.gradient_like(450000, seed=16)
    s3 = oracle.compress(x3, eb, o3)[0]
    o1, o2 = [int(v) for v in s3[64 + 8:64 + 24].view(np.uint64)]
    for pos in (o2 - 40, o1 + 3000, o2 - 20000):
        t = s3.copy(); t[pos] ^= 0x10
        oref, ores, orc = oracle.decompress(t, x3.size, eb)
        rc, r, got = gpu_decompress(nz, t, x3.size, eb, g3)
        assert r["status"] == orc
        assert (got.view(np.uint32) == oref.view(np.uint32)).all(), pos
    # regression: a HUFFMAN frame whose segment table claims zero bits (valid header and code lengths, payload ends
    # after the tables) is rejected at validation, before any bit reader exists
    from crafted import zero_bit_huffman_stream
    step_bits = int(np.float32(oracle.step_constants(eb)[0]).view(np.uint32))
    for n0 in (1, 300, 5000):
        t = zero_bit_huffman_stream(n0, step_bits)
        oref, ores, orc = oracle.decompress(t, n0, eb)
        rc, r, got = gpu_decompress(nz, t, n0, eb, nz.make_opts(chunk_elems=n0))
        assert orc == oracle.ERR_CORRUPT and r["status"] == nz.ERR_CORRUPT and not got.any()
    # the same garbage through the reduce passes (as operand A, as operand B, and as the ring step's incoming stream)
    go = oracle.make_opts(chunk_elems=16384)
    for _ in range(20):
        t = s.copy()
        i = int(rng.integers(off + 32, s.size))
        t[i] ^= int(rng.integers(1, 256))
        for a, b in ((t, s), (s, t)):
            ored, ores, orc = oracle.reduce_frames(a, b, x.size, eb, go)
            rc, r, got = gpu_reduce(nz, a, b, x.size, eb, g)
            assert r["status"] == orc, (i, r, orc)
            if orc == 0:
                assert r["bytes"] == ores.bytes and _first_diff(got, ored) == -1
        ored, ores, orc = oracle.reduce_local(t, x, eb, go)
        rc, r, got = gpu_reduce_local(nz, t, x, eb, g)
        assert r["status"] == orc, (i, r, orc)
        if orc == 0:
            assert r["bytes"] == ores.bytes and _first_diff(got, ored) == -1


# ------------------------------------------------------------------------------------------------
# fused reduce
# ------------------------------------------------------------------------------------------------

def test_reduce_matches_oracle_and_chains(nz):
    n, eb = 300000, 1e-5
    kw = dict(chunk_elems=65536)
    g, o = _opts_pair(nz, **kw)
    msgs = W.peer_messages(n, peers=4, seed0=40)
    streams = [oracle.compress(m, eb, o)[0] for m in msgs]
    acc_o = streams[0]
    acc_g = streams[0]
    for p in range(1, 4):
        acc_o, ores, orc = oracle.reduce_frames(acc_o, streams[p], n, eb, o)
        rc, r, acc_g = gpu_reduce(nz, acc_g, streams[p], n, eb, g)
        assert rc == 0 and orc == 0 and r["status"] == 0
        assert r["bytes"] == ores.bytes and _first_diff(acc_g, acc_o) == -1
        assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    rc, r, got = gpu_decompress(nz, acc_g, n, eb, g)
    true = sum(m.astype(np.float64) for m in msgs)
    assert (np.abs(got.astype(np.float64) - true) <= 4 * float(np.float32(eb))).all()


@pytest.mark.parametrize("wide", [False, True], ids=["plain", "wide_codes"])
def test_reduce_large_frames(nz, wide):
    """1 MiB frames: whole 131072-element blocks take the vectorised add path, the ragged last frame the general
    one; `wide` plants codes that need more than 16 bits after the first reduction (spill array, markers)."""
    n, eb = 2 * 262144 + 70001, 1e-4
    g, o = _opts_pair(nz, chunk_elems=262144)
    msgs = [W.gradient_like(n, seed=90 + p) for p in range(3)]
    if wide:
        step = oracle.step_constants(eb)[0]
        for p, m in enumerate(msgs):
            m[[11, 65536 + 3, 200000, 262144 + 131072 + 5, n - 2]] = np.float32(30000.0 + p) * step   # sums pass 32767
            m[[70000, 262144 + 7]] = np.float32(-(29000.0 + p)) * step
    streams = [oracle.compress(m, eb, o)[0] for m in msgs]
    acc_o = acc_g = streams[0]
    for p in (1, 2):
        acc_o, ores, orc = oracle.reduce_frames(acc_o, streams[p], n, eb, o)
        rc, r, acc_g = gpu_reduce(nz, acc_g, streams[p], n, eb, g)
        assert rc == 0 and orc == 0 and r["status"] == 0
        assert r["bytes"] == ores.bytes and _first_diff(acc_g, acc_o) == -1
        assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    rc, r, got = gpu_decompress(nz, acc_g, n, eb, g)
    ref = oracle.decompress(acc_o, n, eb)[0]
    assert r["status"] == 0 and (got.view(np.uint32) == ref.view(np.uint32)).all()


@pytest.mark.parametrize("ca,cb", [(0, 0), (0, 1), (0, 2), (1, 1), (1, 2), (2, 1), (2, 2), (2, 0)])
def test_reduce_all_codec_pairs(nz, ca, cb):
    n, eb = 70001, 1e-4
    a = W.gradient_like(n, seed=80)
    b = W.sweep_payload("uniform", n, 81)
    sa = oracle.compress(a, eb, oracle.make_opts(chunk_elems=20000, force_codec=ca))[0]
    sb = oracle.compress(b, eb, oracle.make_opts(chunk_elems=20000, force_codec=cb))[0]
    g, o = _opts_pair(nz, chunk_elems=20000)
    ref, ores, orc = oracle.reduce_frames(sa, sb, n, eb, o)
    rc, r, got = gpu_reduce(nz, sa, sb, n, eb, g)
    assert rc == 0 and orc == 0 and r["status"] == 0
    assert r["bytes"] == ores.bytes and _first_diff(got, ref) == -1


@pytest.mark.parametrize("kw", [dict(force_codec=0), dict(min_gain_permil=999), dict(min_gain_permil=650, huff_min_bytes=1 << 20),
                                dict(force_codec=0, predictor=1)])
@pytest.mark.parametrize("n,chunk", [(70001, 20000), (300000, 131072)])
def test_reduce_integer_sums_committed_raw(nz, kw, n, chunk):
    """A frame of integer sums that the selector commits RAW (pinned, gated) holds the fp32 sums of the dequantized
    operands: two streams (incl. wide codes and a RAW operand frame beside it) and the ring step, bytes against the oracle."""
    eb = 1e-4
    pred = kw.get("predictor", 0)
    a = W.gradient_like(n, seed=84)
    b = W.gradient_like(n, seed=85, b=3e-3)
    a[5] = 2.5; a[chunk + 7] = -3.0                              # codes that need more than 16 bits in the staging
    b[n - 3] = np.nan                                            # the last frame of b is RAW
    plain = oracle.make_opts(chunk_elems=chunk, predictor=pred)
    sa = oracle.compress(a, eb, plain)[0]
    sb = oracle.compress(b, eb, plain)[0]
    g, o = _opts_pair(nz, chunk_elems=chunk, **kw)
    ref, ores, orc = oracle.reduce_frames(sa, sb, n, eb, o)
    rc, r, got = gpu_reduce(nz, sa, sb, n, eb, g)
    assert rc == 0 and orc == 0 and r["status"] == 0 and ores.n_raw > 1
    assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    assert r["bytes"] == ores.bytes and _first_diff(got, ref) == -1
    ref, ores, orc = oracle.reduce_local(sa, b, eb, o)
    rc, r, got = gpu_reduce_local(nz, sa, b, eb, g)
    assert rc == 0 and orc == 0 and r["status"] == 0 and ores.n_raw > 1
    assert r["bytes"] == ores.bytes and _first_diff(got, ref) == -1


def test_reduce_raw_nan_overflow_and_mismatch(nz):
    n, eb = 3000, 1e-3
    g, o = _opts_pair(nz, chunk_elems=1000)
    a = W.gradient_like(n, seed=70); b = W.gradient_like(n, seed=71)
    a[1500] = np.nan; b[2500] = np.inf; a[2501] = -np.inf
    sa = oracle.compress(a, eb, o)[0]; sb = oracle.compress(b, eb, o)[0]
    ref, ores, orc = oracle.reduce_frames(sa, sb, n, eb, o)
    rc, r, got = gpu_reduce(nz, sa, sb, n, eb, g)
    assert orc == 0 and r["status"] == 0 and r["bytes"] == ores.bytes and _first_diff(got, ref) == -1
    # double a stream until a sum passes 2^30: that frame is committed as RAW with fp32 sums, the others stay coded
    x = W.gradient_like(3000, seed=72)
    x[:1000] = 0.0
    x[7] = np.float32(32767.0) * oracle.step_constants(eb)[0]
    s = oracle.compress(x, eb, o)[0]
    for i in range(17):
        s_o, ores, orc = oracle.reduce_frames(s, s, 3000, eb, o)
        rc, r, s_g = gpu_reduce(nz, s, s, 3000, eb, g)
        assert orc == 0 and r["status"] == 0 and r["bytes"] == ores.bytes and _first_diff(s_g, s_o) == -1, i
        assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
        s = s_o
    assert ores.n_raw == 1
    # operands that disagree
    sc = oracle.compress(a, 2e-3, o)[0]
    assert gpu_reduce(nz, sa, sc, n, eb, g)[1]["status"] == nz.ERR_MISMATCH
    sd = oracle.compress(a, eb, oracle.make_opts(chunk_elems=500))[0]
    assert gpu_reduce(nz, sa, sd, n, eb, g)[1]["status"] == nz.ERR_MISMATCH
    t = sa.copy(); t[int(t[64:72].view(np.uint64)[0]) + 4] ^= 7          # frame 0 codec id
    assert gpu_reduce(nz, t, sb, n, eb, g)[1]["status"] == nz.ERR_CORRUPT
    # capacity
    rc, r, _ = gpu_reduce(nz, sa, sb, n, eb, g, cap=int(ores.bytes) - 16)
    assert r["status"] == nz.ERR_CAPACITY and r["bytes"] == 0


# ------------------------------------------------------------------------------------------------
# seeded sweep over sizes, frame lengths, alphabets, bounds and value mixtures
# ------------------------------------------------------------------------------------------------

def _mixture(rng, n):
    """Values with the structure the method meets: a peaked body, heavy outliers, runs of zeros, smooth stretches."""
    kind = rng.integers(0, 5)
    if kind == 0:
        x = rng.laplace(0, 1e-3, n)
    elif kind == 1:
        x = rng.laplace(0, 1e-3, n)
        m = rng.random(n) < rng.choice([0.001, 0.02, 0.2])
        x[m] = rng.laplace(0, rng.choice([0.05, 1.0, 30.0]), int(m.sum()))
    elif kind == 2:
        x = np.sin(np.arange(n) * rng.uniform(1e-4, 1e-2)) * rng.uniform(1e-3, 1.0) + rng.normal(0, 1e-4, n)
    elif kind == 3:
        x = rng.uniform(-1, 1, n) * rng.choice([1e-3, 0.1, 5.0])
    else:
        x = rng.laplace(0, 1e-3, n)
        a = rng.integers(0, n)
        x[a:a + rng.integers(0, n)] = 0.0
    return x.astype(np.float32)


@pytest.mark.parametrize("seed", range(24))
def test_seeded_sweep(nz, seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.choice([1, 5, 255, 256, 257, 4097, 65535, 65536, 65537, 131072, 200001, 300007, 600011]))
    chunk = int(rng.choice([16, 1000, 4096, 16384, 65536, 100003, 131072, 262144, 1 << 20]))
    K = int(rng.choice([2, 4, 64, 256, 256, 256, 512, 1024]))
    eb = float(rng.choice([1e-2, 1e-3, 1e-4, 1e-5]))
    kw = dict(chunk_elems=chunk, alphabet=K)
    if rng.random() < 0.2:
        kw["force_codec"] = int(rng.integers(0, 3))
    a, b = _mixture(rng, n), _mixture(rng, n)
    if rng.random() < 0.15:
        a[rng.integers(0, n)] = np.nan
    ref_a, _ = check_compress(nz, a, eb, **kw)
    check_decompress(nz, ref_a, a, eb, **kw)
    g, o = _opts_pair(nz, **kw)
    ref_b = oracle.compress(b, eb, o)[0]
    ref, ores, orc = oracle.reduce_frames(ref_a, ref_b, n, eb, o)
    rc, r, got = gpu_reduce(nz, ref_a, ref_b, n, eb, g)
    assert rc == 0 and r["status"] == orc
    if orc == 0:
        assert r["bytes"] == ores.bytes and _first_diff(got, ref) == -1
        ref2, ores2, orc2 = oracle.reduce_frames(ref, ref_a, n, eb, o)          # a second level: wider codes
        rc, r2, got2 = gpu_reduce(nz, got, ref_a, n, eb, g)
        assert r2["status"] == orc2
        if orc2 == 0:
            assert r2["bytes"] == ores2.bytes and _first_diff(got2, ref2) == -1


# ------------------------------------------------------------------------------------------------
# the remaining workload shapes (C3, C4, C5) at sizes the oracle finishes in seconds, and C2 at full size
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("rel", [1e-2, 1e-3, 1e-4])
def test_c3_random_field_bound_sweep(nz, rel):
    x = W.gaussian_random_field(N=64, seed=3)                      # 262144 elements, P(k) ~ k^-3, unit variance
    eb = W.abs_bound_from_rel(x, rel)
    ref, _ = check_compress(nz, x, eb, chunk_elems=65536)
    check_decompress(nz, ref, x, eb, chunk_elems=65536)


def test_c4_ring_step_chain_and_association_order(nz):
    n, eb = 200000, 1e-5
    g, o = _opts_pair(nz, chunk_elems=65536)
    msgs = W.peer_messages(n, peers=8, seed0=40)
    streams = [oracle.compress(m, eb, o)[0] for m in msgs]

    def chain(order):
        acc = streams[order[0]]
        for p in order[1:]:
            rc, r, acc = gpu_reduce(nz, acc, streams[p], n, eb, g)
            assert rc == 0 and r["status"] == 0
        return acc
    a = chain(list(range(8)))
    b = chain([7, 3, 0, 5, 1, 6, 2, 4])
    acc_o = streams[0]
    for p in range(1, 8):
        acc_o = oracle.reduce_frames(acc_o, streams[p], n, eb, o)[0]
    assert _first_diff(a, acc_o) == -1 and _first_diff(b, acc_o) == -1       # 7 steps, any order: identical bytes
    rc, r, got = gpu_decompress(nz, a, n, eb, g)
    true = sum(m.astype(np.float64) for m in msgs)
    assert (np.abs(got.astype(np.float64) - true) <= 8 * float(np.float32(eb))).all()


@pytest.mark.parametrize("kind", ["uniform", "laplace", "sinusoid"])
@pytest.mark.parametrize("n", [16384, 65536, 262144, 1048576])
def test_c5_size_sweep(nz, kind, n):
    x = W.sweep_payload(kind, n, 50)
    chunk = 16384 if 4 * n <= (4 << 20) else 262144
    ref, _ = check_compress(nz, x, 1e-4, chunk_elems=chunk)
    check_decompress(nz, ref, x, 1e-4, chunk_elems=chunk)


def test_c2_full_size(nz):
    """The headline message (64 Mi fp32, 1 MiB frames) in the configuration bench.py times: compressed stream,
    decompressed values and the reduced stream against the oracle, whole message."""
    import torch
    n = 1 << 26
    x = W.gradient_like(n, seed=2)
    peer = W.gradient_like(n, seed=102)
    eb = float(np.float32(W.abs_bound_from_rel(x, 1e-4)))
    g, o = _opts_pair(nz, chunk_elems=262144)
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    rc, out = sess.compress(torch.from_numpy(x).to("cuda:0"), eb)
    r = sess.result()
    ref, ores, orc = oracle.compress(x, eb, o)
    assert rc == 0 and orc == 0 and r["status"] == 0 and r["bytes"] == ores.bytes
    assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    assert _first_diff(out[:r["bytes"]].cpu().numpy(), ref) == -1
    nbytes = r["bytes"]
    rc, y = sess.decompress(out, nbytes, n, eb)
    assert rc == 0 and sess.result()["status"] == 0
    yo = oracle.decompress(ref, n, eb)[0]
    y = y.cpu().numpy()
    assert (y.view(np.uint32) == yo.view(np.uint32)).all()
    assert float(np.max(np.abs(y.astype(np.float64) - x.astype(np.float64)))) <= float(np.float32(eb))
    del y, yo
    rc, pout = nz.Session(n, g, "cuda:0").compress(torch.from_numpy(peer).to("cuda:0"), eb)
    pref = oracle.compress(peer, eb, o)[0]
    rc, red = sess.reduce(out, nbytes, pout, pref.size, n, eb)
    rr = sess.result()
    ro, rres, rrc = oracle.reduce_frames(ref, pref, n, eb, o)
    assert rc == 0 and rrc == 0 and rr["status"] == 0 and rr["bytes"] == rres.bytes
    assert _first_diff(red[:rr["bytes"]].cpu().numpy(), ro) == -1


# ------------------------------------------------------------------------------------------------
# ring-step reduce: incoming frames + the rank's own fp32 data
# ------------------------------------------------------------------------------------------------

def _check_reduce_local(nz, a_stream, x, eb, **kw):
    g, o = _opts_pair(nz, **kw)
    ref, ores, orc = oracle.reduce_local(a_stream, x, eb, o)
    rc, r, got = gpu_reduce_local(nz, a_stream, x, eb, g)
    assert rc == 0 and r["status"] == orc, (r, orc)
    if orc == 0:
        assert r["bytes"] == ores.bytes and _first_diff(got, ref) == -1
        assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    else:
        assert r["bytes"] == 0
    return ref


def test_reduce_local_ring_chain(nz):
    """A reduce-scatter ring as one rank sees it: every step adds the rank's own fp32 data to the incoming frames."""
    n, eb = 2 * 262144 + 70001, 1e-5
    kw = dict(chunk_elems=262144)
    msgs = W.peer_messages(n, peers=4, seed0=40)
    acc = oracle.compress(msgs[0], eb, oracle.make_opts(**kw))[0]
    for p in (1, 2, 3):
        acc = _check_reduce_local(nz, acc, msgs[p], eb, **kw)
    g, _ = _opts_pair(nz, **kw)
    rc, r, got = gpu_decompress(nz, acc, n, eb, g)
    true = sum(m.astype(np.float64) for m in msgs)
    assert (np.abs(got.astype(np.float64) - true) <= 4 * float(np.float32(eb))).all()


@pytest.mark.parametrize("case", ["local_nan", "incoming_raw", "both", "fixedlen_in", "raw_forced", "wide_sums"])
def test_reduce_local_frame_kinds(nz, case):
    n, eb = 2 * 131072 + 9001, 1e-4
    kw = dict(chunk_elems=131072)
    a, x = W.gradient_like(n, seed=81), W.gradient_like(n, seed=82)
    in_kw = dict(kw)
    if case in ("local_nan", "both"):
        x[[5, 131072 + 70000]] = [np.nan, 3e38]           # frames 0 and 1 of the local data cannot be quantized
    if case in ("incoming_raw", "both"):
        a[[131072 + 1, n - 1]] = [np.inf, -np.inf]        # frames 1 and 2 of the incoming stream are RAW
    if case == "fixedlen_in":
        in_kw["force_codec"] = 1
    if case == "raw_forced":
        in_kw["force_codec"] = 0
    if case == "wide_sums":
        step = oracle.step_constants(eb)[0]
        a[[3, 70000, 131072 + 5]] = np.float32(30000.0) * step
        x[[3, 70000, 131072 + 5]] = np.float32(31000.0) * step
        x[9] = np.float32(-32767.0) * step; a[9] = np.float32(-32767.0) * step
    sa = oracle.compress(a, eb, oracle.make_opts(**in_kw))[0]
    _check_reduce_local(nz, sa, x, eb, **kw)


def test_reduce_local_overflow_mismatch_capacity(nz):
    eb = 1e-3
    g, o = _opts_pair(nz, chunk_elems=1000)
    step = oracle.step_constants(eb)[0]
    z = np.zeros(1000, np.float32); z[7] = np.float32(32767.0) * step
    s = oracle.compress(z, eb, o)[0]
    for _ in range(15):
        s = oracle.reduce_frames(s, s, 1000, eb, o)[0]
    s1 = _check_reduce_local(nz, s, z, eb, chunk_elems=1000)                      # 2^30 - 1: still carried
    s2 = _check_reduce_local(nz, s1, z, eb, chunk_elems=1000)                     # past 2^30: the frame is committed as RAW
    assert oracle.decode_codes(s2, 1000, eb)[2].tolist() == [1]
    _check_reduce_local(nz, s2, z, eb, chunk_elems=1000)                          # and stays RAW
    zn = z.copy(); zn[500] = np.nan                                              # the local data turns the frame RAW anyway
    _check_reduce_local(nz, s1, zn, eb, chunk_elems=1000)
    # several frames, one of them overflowing in its second half only
    big = W.gradient_like(300000, seed=73)
    gk, ok = _opts_pair(nz, chunk_elems=140000)
    big[140000 + 70000] = np.float32(32767.0) * step
    sb = oracle.compress(big, eb, ok)[0]
    for _ in range(15):
        sb = oracle.reduce_frames(sb, sb, big.size, eb, ok)[0]
    sb1 = _check_reduce_local(nz, sb, big, eb, chunk_elems=140000)
    sb2 = _check_reduce_local(nz, sb1, big, eb, chunk_elems=140000)
    assert oracle.decode_codes(sb2, big.size, eb)[2].tolist() == [0, 1, 0]
    ref, ores, orc = oracle.reduce_frames(sb1, sb, big.size, eb, ok)
    rc, r, got = gpu_reduce(nz, sb1, sb, big.size, eb, gk)
    assert orc == 0 and r["status"] == 0 and ores.n_raw == 1 and _first_diff(got, ref) == -1
    a = W.gradient_like(3000, seed=70)
    sa = oracle.compress(a, eb, o)[0]
    assert gpu_reduce_local(nz, sa, a, 2e-3, g)[1]["status"] == nz.ERR_MISMATCH
    g2 = nz.make_opts(chunk_elems=500)
    assert gpu_reduce_local(nz, sa, a, eb, g2)[1]["status"] == nz.ERR_MISMATCH
    ref, ores, _ = oracle.reduce_local(sa, a, eb, o)
    rc, r, _ = gpu_reduce_local(nz, sa, a, eb, g, cap=int(ores.bytes) - 16)
    assert r["status"] == nz.ERR_CAPACITY and r["bytes"] == 0
    # a broken stream header, a truncated stream
    t = sa.copy(); t[0] ^= 1
    assert oracle.reduce_local(t, a, eb, o)[2] == oracle.ERR_CORRUPT
    rc, r, _ = gpu_reduce_local(nz, t, a, eb, g)
    assert r["status"] == nz.ERR_CORRUPT and r["bytes"] == 0
    rc, r, _ = gpu_reduce_local(nz, sa[:-16], a, eb, g)
    assert r["status"] == oracle.reduce_local(sa[:-16], a, eb, o)[2] == nz.ERR_CORRUPT and r["bytes"] == 0


@pytest.mark.parametrize("seed", range(12))
def test_reduce_local_seeded_sweep(nz, seed):
    rng = np.random.default_rng(3000 + seed)
    n = int(rng.choice([1, 257, 4097, 65537, 131072, 200001, 600011]))
    chunk = int(rng.choice([16, 1000, 16384, 65536, 100003, 131072, 262144]))
    K = int(rng.choice([2, 64, 256, 256, 1024]))
    eb = float(rng.choice([1e-3, 1e-4, 1e-5]))
    kw = dict(chunk_elems=chunk, alphabet=K)
    a, x = _mixture(rng, n), _mixture(rng, n)
    if rng.random() < 0.25:
        x[rng.integers(0, n)] = np.nan
    if rng.random() < 0.25:
        a[rng.integers(0, n)] = np.inf
    sa = oracle.compress(a, eb, oracle.make_opts(**kw))[0]
    s1 = _check_reduce_local(nz, sa, x, eb, **kw)
    if s1.size:
        _check_reduce_local(nz, s1, a, eb, **kw)                                  # second ring step on wider codes


@pytest.mark.parametrize("seed", range(8))
def test_codebook_tie_heavy_histograms(nz, seed):
    """Small frames of few equally likely codes: counts tie all the time, internal nodes tie with leaves, and the
    merge alternates between long leaf-pair and node-pair runs -- the cases the run-at-a-time merge must get exactly
    like the sequential two-queue rule (a leaf wins a tie)."""
    rng = np.random.default_rng(5000 + seed)
    eb = 1e-3
    step = oracle.step_constants(eb)[0]
    levels = int(rng.choice([2, 3, 5, 8, 17, 33, 100, 200]))
    chunk = int(rng.choice([64, 256, 1000, 4096]))
    n = chunk * int(rng.integers(3, 40)) + int(rng.integers(0, chunk))
    q = rng.integers(-levels, levels + 1, n)
    if seed % 2:
        q = np.repeat(np.arange(-levels, levels + 1), n // (2 * levels + 1) + 1)[:n]      # exactly equal counts
        rng.shuffle(q)
    x = (q.astype(np.float32) * np.float32(step)).astype(np.float32)
    K = int(rng.choice([16, 64, 256, 1024]))
    ref, _ = check_compress(nz, x, eb, chunk_elems=chunk, alphabet=K, force_codec=2)
    check_decompress(nz, ref, x, eb, chunk_elems=chunk, alphabet=K)


@pytest.mark.parametrize("shape", ["equal", "near_equal", "fibonacci", "staircase", "spikes", "dyadic", "few_heavy_many_light"])
@pytest.mark.parametrize("K", [256, 1024])
def test_codebook_histogram_shapes_in_maximal_frames(nz, shape, K):
    """Histograms chosen for the code construction's merge, in frames of the maximal size (2^20 symbols, so weights
    reach 2^20): hundreds of equal counts (long runs of leaf pairs, windows that overflow), near-equal counts, a
    Fibonacci chain (a node joins a leaf at every step, deepest codes), stairs of equal counts (ties between leaves
    and nodes of the same weight), a few heavy symbols over a flat tail, dyadic counts.  HUFFMAN pinned, bytes
    against the oracle, then decompress."""
    rng = np.random.default_rng(7000 + K + len(shape))
    nsym = K - 2                                               # symbols z = 0 .. K-3 (no escapes)
    n = 1 << 20
    if shape == "equal":
        c = np.full(nsym, n // nsym)
    elif shape == "near_equal":
        c = (n / nsym * (1 + 0.01 * rng.standard_normal(nsym))).astype(np.int64)
    elif shape == "fibonacci":
        f = [1, 1]
        while sum(f) + f[-1] + f[-2] <= n and len(f) < nsym:
            f.append(f[-1] + f[-2])
        c = np.array(f)
    elif shape == "staircase":
        c = np.repeat(np.arange(1, nsym // 37 + 2) * 13, 37)[:nsym]
    elif shape == "spikes":
        c = np.full(nsym, 50); c[:3] = [n // 3, n // 5, n // 9]
    elif shape == "dyadic":
        c = np.array([1 << (18 - min(i // 2, 18)) for i in range(min(nsym, 60))])
    else:
        c = np.concatenate([np.full(5, n // 8), np.full(nsym - 5, 300)])
    c = np.maximum(c, 0).astype(np.int64)
    scale = min(1.0, n / c.sum())
    if scale < 1.0:
        c = np.maximum((c * scale).astype(np.int64), 1)
    z = np.repeat(np.arange(c.size), c)
    rng.shuffle(z)
    tail = z[:50000]                                           # a second, ragged frame
    z = np.concatenate([z, tail])
    q = np.where(z & 1, -((z + 1) >> 1), z >> 1).astype(np.int64)
    eb = 1e-3
    step = oracle.step_constants(eb)[0]
    x = (q.astype(np.float32) * np.float32(step)).astype(np.float32)
    assert (oracle.quantize(x, eb)[0] == q).all()
    ref, ores = check_compress(nz, x, eb, chunk_elems=1 << 20, alphabet=K, force_codec=2)
    assert ores.n_huff == ores.n_frames
    check_decompress(nz, ref, x, eb, chunk_elems=1 << 20, alphabet=K)


def test_more_than_2_to_31_elements(nz):
    """Index arithmetic past 32 bits: 2^31 + 70001 elements (8.6 GB of fp32).  Too large for the oracle to hold, so
    the check is by properties that hold at any size: frame count, stream header, |x - xhat| <= eb for every element,
    a decoded stream of the expected length, and byte-identity of the first and last frames with the oracle's
    encoding of the same frames."""
    import torch
    n = (1 << 31) + 70001
    chunk = 1 << 20
    eb = 1e-4
    g = nz.make_opts(chunk_elems=chunk)
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(7)
    x = torch.empty(n, dtype=torch.float32, device="cuda:0")
    x.normal_(0.0, 1e-3, generator=gen)
    sess = nz.Session(n, g, "cuda:0")
    rc, out = sess.compress(x, eb)
    r = sess.result()
    nfr = (n + chunk - 1) // chunk
    assert rc == 0 and r["status"] == 0 and r["n_frames"] == nfr and r["n_raw"] == 0
    hdr = out[:64].cpu().numpy()
    assert int(hdr[8:16].view(np.uint64)[0]) == n and int(hdr[40:48].view(np.uint64)[0]) == r["bytes"]
    offs = out[64:64 + 8 * nfr].cpu().numpy().view(np.uint64).astype(np.int64)
    assert (np.diff(offs) > 0).all() and offs[-1] < r["bytes"]
    # first and last frame against the oracle's frame encoder
    o = oracle.make_opts(chunk_elems=chunk)
    step_bits = int(np.float32(oracle.step_constants(eb)[0]).view(np.uint32))
    for k in (0, nfr - 1):
        xf = x[k * chunk:min(n, (k + 1) * chunk)].cpu().numpy()
        q, ok = oracle.quantize(xf, eb)
        assert ok.all()
        plan = oracle.frame_plan(q, o)
        fr = oracle.frame_encode(q, plan["codec"], o, step_bits=step_bits)
        got = out[int(offs[k]):int(offs[k]) + fr.size].cpu().numpy()
        assert (got == fr).all()
    y = torch.empty_like(x)
    rc, y = sess.decompress(out, r["bytes"], n, eb, out=y)
    r2 = sess.result()
    assert rc == 0 and r2["status"] == 0 and r2["bytes"] == r["bytes"] and r2["n_huff"] + r2["n_fixed"] == nfr
    err = (y.double() - x.double()).abs_().max().item()
    assert err <= float(np.float32(eb))


def test_calls_can_be_captured_in_a_hip_graph(nz):
    """The entry points only launch kernels (no allocation, no memset, no synchronisation), so a caller may record
    them into a HIP graph.  Replays -- with eager work and synchronisations in between -- must reproduce the eager
    result every time."""
    import torch
    n, eb = 300000, 1e-4
    g, o = _opts_pair(nz, chunk_elems=65536)
    x = W.gradient_like(n, seed=21)
    peer = oracle.compress(W.gradient_like(n, seed=22), eb, o)[0]
    ref = oracle.compress(x, eb, o)[0]
    ref_red = oracle.reduce_frames(ref, peer, n, eb, o)[0]
    dx = _to_dev(nz, x)
    dpeer = _to_dev(nz, np.concatenate([peer, np.zeros((-peer.size) % 16, np.uint8)]))
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    res_c = torch.zeros(nz.RESULT_BYTES, dtype=torch.uint8, device="cuda:0")
    res_r = torch.zeros(nz.RESULT_BYTES, dtype=torch.uint8, device="cuda:0")
    out, red = sess.new_stream_buffer(), sess.new_stream_buffer()
    y = torch.empty(n, dtype=torch.float32, device="cuda:0")

    def work():
        assert nz.nz_compress(dx, n, eb, out, sess.cap, res_c, g, sess.ws, sess.ws_bytes) == 0
        assert nz.nz_decompress(out, ref.size, y, n, eb, sess.res, g, sess.ws, sess.ws_bytes) == 0
        assert nz.nz_reduce_frames(out, ref.size, dpeer, peer.size, red, sess.cap, n, eb, res_r, g, sess.ws, sess.ws_bytes) == 0

    work()                                            # eager, also warms everything up
    torch.cuda.synchronize()
    y_ref = oracle.decompress(ref, n, eb)[0]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        work()
        graph.capture_end()
    for rep in range(3):
        out.zero_(); red.zero_(); y.zero_(); res_c.zero_(); res_r.zero_()      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        rc_, rr_ = nz.read_result(res_c), nz.read_result(res_r)
        assert rc_["status"] == 0 and rc_["bytes"] == ref.size and rr_["status"] == 0 and rr_["bytes"] == ref_red.size
        assert _first_diff(out[:ref.size].cpu().numpy(), ref) == -1, rep
        assert _first_diff(red[:ref_red.size].cpu().numpy(), ref_red) == -1, rep
        assert (y.cpu().numpy().view(np.uint32) == y_ref.view(np.uint32)).all(), rep


def test_calls_on_two_streams_with_their_own_buffers_run_side_by_side(nz):
    """Two calls may overlap in time when they share nothing but read-only inputs: each stream here has its own
    workspace, output and result record (the library keeps no state).  Both results must be the oracle's, run after
    run."""
    import torch
    n, eb = 700000, 1e-4
    g, o = _opts_pair(nz, chunk_elems=65536)
    xs = [W.gradient_like(n, seed=31), W.sweep_payload("uniform", n, 32)]
    refs = [oracle.compress(x, eb, o)[0] for x in xs]
    ref_red = oracle.reduce_frames(refs[0], refs[1], n, eb, o)[0]
    dxs = [_to_dev(nz, x) for x in xs]
    sess = [nz.Session(n, g, "cuda:0", reduce=True) for _ in range(2)]
    outs = [s_.new_stream_buffer() for s_ in sess]
    ys = [torch.empty(n, dtype=torch.float32, device="cuda:0") for _ in range(2)]
    reds = [s_.new_stream_buffer() for s_ in sess]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]                 # default priority
    torch.cuda.synchronize()
    for rep in range(4):
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                st = streams[k]
                assert nz.nz_compress(dxs[k], n, eb, outs[k], sess[k].cap, sess[k].res, g, sess[k].ws, sess[k].ws_bytes, stream=st) == 0
        torch.cuda.synchronize()
        for k in range(2):
            r = sess[k].result()
            assert r["status"] == 0 and r["bytes"] == refs[k].size and _first_diff(outs[k][:r["bytes"]].cpu().numpy(), refs[k]) == -1, (rep, k)
        # a decompress of stream 0 beside a reduce of both
        with torch.cuda.stream(streams[0]):
            assert nz.nz_decompress(outs[0], refs[0].size, ys[0], n, eb, sess[0].res, g, sess[0].ws, sess[0].ws_bytes,
                                    stream=streams[0]) == 0
        with torch.cuda.stream(streams[1]):
            assert nz.nz_reduce_frames(outs[0], refs[0].size, outs[1], refs[1].size, reds[1], sess[1].cap, n, eb, sess[1].res, g,
                                       sess[1].ws, sess[1].ws_bytes, stream=streams[1]) == 0
        torch.cuda.synchronize()
        assert sess[0].result()["status"] == 0 and sess[1].result()["status"] == 0
        assert (ys[0].cpu().numpy().view(np.uint32) == oracle.decompress(refs[0], n, eb)[0].view(np.uint32)).all(), rep
        assert _first_diff(reds[1][:ref_red.size].cpu().numpy(), ref_red) == -1, rep


# ------------------------------------------------------------------------------------------------
# exact ties, deepest codes, many second-level tables, refused options
# ------------------------------------------------------------------------------------------------

def test_exact_ties_round_to_even(nz):
    """eb = fl32(32/63) makes step and 1/step exactly 1.0, so x = k + 1/2 is an exact tie (the golden rows of the CPU
    pin); a whole message of such ties and near-ties must give the oracle's bytes."""
    eb = float(np.float32(32.0 / 63.0))
    rng = np.random.default_rng(77)
    k = rng.integers(-2000, 2000, 100000)
    x = (k + 0.5).astype(np.float32)
    x[::7] = np.nextafter(x[::7], np.float32(np.inf))            # just above a tie
    x[3::7] = np.nextafter(x[3::7], np.float32(-np.inf))         # just below
    rows = [l.split() for l in open(__file__.replace("test_gpu_parity.py", "golden/quantizer_ties.txt")) if l.strip() and l[0] != "#"]
    x[:len(rows)] = [float(r[0]) for r in rows]
    ref, _ = check_compress(nz, x, eb, chunk_elems=16384, alphabet=1024)
    g, _ = _opts_pair(nz, chunk_elems=16384, alphabet=1024)
    rc, r, got = gpu_decompress(nz, ref, x.size, eb, g)
    assert r["status"] == 0 and got[:len(rows)].tolist() == [float(r_[2]) for r_ in rows]
    check_decompress(nz, ref, x, eb, chunk_elems=16384, alphabet=1024)


def _fibonacci_codes(adjacent_rare=True):
    fib = [1, 1]
    while len(fib) < 28:
        fib.append(fib[-1] + fib[-2])
    rng = np.random.default_rng(5)
    z = np.concatenate([np.full(c, i) for i, c in enumerate(fib)])            # zigzag code i occurs fib[i] times
    head, tail = z[:sum(fib[:8])], z[sum(fib[:8]):]
    rng.shuffle(tail)
    z = np.concatenate([head, tail]) if adjacent_rare else rng.permutation(z)  # the rarest (27-bit) codes side by side
    return ((z >> 1) ^ -(z & 1)).astype(np.int32)


@pytest.mark.parametrize("K", [32, 256])
def test_deepest_codes_fibonacci_histogram(nz, K):
    """Fibonacci counts give the deepest optimal code a 2^20-symbol frame can have (27 bits): the decoder's
    range-compare path and the encoder's more-than-64-bits-per-thread path at their limit, through compress,
    decompress, both reduces (the sums 2q keep the Fibonacci histogram)."""
    q = _fibonacci_codes()
    eb = float(np.float32(32.0 / 63.0))                                       # step = 1: x = q exactly
    x = q.astype(np.float32)
    kw = dict(chunk_elems=1 << 20, alphabet=K)
    plan = oracle.frame_plan(q, oracle.make_opts(**kw))
    assert plan["len"].max() == 27 and plan["codec"] == oracle.HUFFMAN
    ref, _ = check_compress(nz, x, eb, **kw)
    check_decompress(nz, ref, x, eb, **kw)
    g, o = _opts_pair(nz, **kw)
    red, ores, orc = oracle.reduce_frames(ref, ref, x.size, eb, o)
    rc, r, got = gpu_reduce(nz, ref, ref, x.size, eb, g)
    assert orc == 0 and r["status"] == 0 and r["bytes"] == ores.bytes and _first_diff(got, red) == -1
    check_decompress(nz, red, 2 * x, eb, **kw)
    _check_reduce_local(nz, ref, x, eb, **kw)
    # and a second message with the symbols in another order as operand B
    x2 = _fibonacci_codes(adjacent_rare=False).astype(np.float32)
    ref2, _ = check_compress(nz, x2, eb, **kw)
    red, ores, orc = oracle.reduce_frames(ref, ref2, x.size, eb, o)
    rc, r, got = gpu_reduce(nz, ref, ref2, x.size, eb, g)
    assert orc == 0 and r["status"] == 0 and _first_diff(got, red) == -1


def test_more_than_32_second_level_tables(nz):
    """K = 1024 with four heavy symbols and a thousand equally rare ones: the rare codes are 13-14 bits long and start
    with some 200 different 11-bit prefixes, far more than the 32 second-level tables the decoder keeps."""
    rng = np.random.default_rng(6)
    n = 1 << 20
    z = rng.integers(0, 4, n)
    rare = rng.random(n) < 0.1
    z[rare] = rng.integers(4, 1023, int(rare.sum()))
    q = ((z >> 1) ^ -(z & 1)).astype(np.int32)
    eb = float(np.float32(32.0 / 63.0))
    x = q.astype(np.float32)
    kw = dict(chunk_elems=1 << 20, alphabet=1024)
    plan = oracle.frame_plan(q, oracle.make_opts(**kw))
    long_codes = [(int(c) >> (int(l) - 11)) for c, l in zip(plan["code"], plan["len"]) if l > 11]
    assert len(set(long_codes)) > 100 and plan["codec"] == oracle.HUFFMAN
    ref, _ = check_compress(nz, x, eb, **kw)
    check_decompress(nz, ref, x, eb, **kw)
    g, o = _opts_pair(nz, **kw)
    red, ores, orc = oracle.reduce_frames(ref, ref, n, eb, o)
    rc, r, got = gpu_reduce(nz, ref, ref, n, eb, g)
    assert orc == 0 and r["status"] == 0 and _first_diff(got, red) == -1
    _check_reduce_local(nz, ref, x, eb, **kw)


def test_pinned_huffman_all_escapes_fits_its_bound(nz):
    """K = 2 and no zero codes: every symbol escapes (33 bits each), more than RAW; the pinned-HUFFMAN capacity bound
    must cover the stream."""
    n = 50000
    x = (np.arange(n) % 7 + 3).astype(np.float32)
    eb = float(np.float32(32.0 / 63.0))
    kw = dict(chunk_elems=16384, alphabet=2, force_codec=2)
    g, o = _opts_pair(nz, **kw)
    ref, ores = check_compress(nz, x, eb, **kw)
    assert ref.size > 4 * n and ref.size <= nz.nz_compress_bound(n, g) == oracle.compress_bound(n, o)
    check_decompress(nz, ref, x, eb, **kw)


@pytest.mark.parametrize("seg", [32, 64, 128, 512, 1024, 255])
def test_other_segment_sizes_are_refused_by_every_entry_point(nz, seg):
    """The format allows 32..1024 symbols per segment (the oracle handles them); these kernels are built around one
    256-symbol segment per wavefront pass and refuse everything else, consistently."""
    import torch
    n, eb = 70000, 1e-4
    x = W.gradient_like(n, seed=9)
    good = nz.make_opts(chunk_elems=16384)
    bad = nz.make_opts(chunk_elems=16384, seg_syms=seg)
    sess = nz.Session(n, good, "cuda:0", reduce=True)
    dx = _to_dev(nz, x)
    rc, out = sess.compress(dx, eb)
    nbytes = sess.result()["bytes"]
    assert rc == 0 and nbytes > 0
    y = torch.empty(n, dtype=torch.float32, device="cuda:0")
    assert nz.nz_compress_bound(n, bad) == 0 and nz.nz_workspace_bytes(n, bad) == 0 and nz.nz_reduce_workspace_bytes(n, bad) == 0
    assert nz.nz_compress(dx, n, eb, out, sess.cap, sess.res, bad, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_decompress(out, nbytes, y, n, eb, sess.res, bad, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    red = sess.new_stream_buffer()
    assert nz.nz_reduce_frames(out, nbytes, out, nbytes, red, sess.cap, n, eb, sess.res, bad, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_reduce_local(out, nbytes, dx, red, sess.cap, n, eb, sess.res, bad, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    # a stream that was written with another segment size (by the oracle) does not match what these kernels decode
    so = oracle.compress(x, eb, oracle.make_opts(chunk_elems=16384, seg_syms=seg))[0]
    rc, r, _ = gpu_decompress(nz, so, n, eb, good)
    assert r["status"] == nz.ERR_MISMATCH
    torch.cuda.synchronize()


@pytest.mark.parametrize("predictor", [0, 1], ids=["plain", "delta"])
def test_fixedlen_every_width_by_doubling(nz, predictor):
    """Pinned FIXEDLEN through a chain of self-reductions: every reduce doubles the codes, so the width grows by one
    bit per step from what the data needs up to 31 (32 with the predictor), until a sum passes 2^30 and its frame
    turns RAW.  Frames of 20000 elements with a ragged tail, so passes end inside a word and inside a 16-byte group."""
    n, eb = 70001, float(np.float32(32.0 / 63.0))                       # step = 1: x = q
    rng = np.random.default_rng(77)
    q = rng.integers(-5, 6, n).astype(np.float32)
    q[[3, 4, 20000, 45000, n - 1]] = [32767.0, -32767.0, -32767.0, 20001.0, -17.0]   # full-range codes, two of them adjacent
    kw = dict(chunk_elems=20000, force_codec=1, predictor=predictor)
    g, o = _opts_pair(nz, **kw)
    acc, ores, orc = oracle.compress(q, eb, o)
    rc, r, got = gpu_compress(nz, q, eb, g)
    assert orc == 0 and r["status"] == 0 and _first_diff(got, acc) == -1
    saw_raw = False
    for step in range(17):
        ref, ores, orc = oracle.reduce_frames(acc, acc, n, eb, o)
        rc, r, got = gpu_reduce(nz, acc, acc, n, eb, g)
        assert orc == 0 and rc == 0 and r["status"] == 0, (step, r)
        assert (r["n_raw"], r["n_fixed"], r["n_huff"], r["bytes"]) == (ores.n_raw, ores.n_fixed, ores.n_huff, ores.bytes), step
        assert _first_diff(got, ref) == -1, (step, _first_diff(got, ref))
        rc, r, y = gpu_decompress(nz, ref, n, eb, g)
        want = oracle.decompress(ref, n, eb)[0]
        assert r["status"] == 0 and (y.view(np.uint32) == want.view(np.uint32)).all(), step
        saw_raw = saw_raw or ores.n_raw > 0
        acc = ref
    assert saw_raw                                                      # 32767 * 2^16 > 2^30: the chain reached the RAW fallback
