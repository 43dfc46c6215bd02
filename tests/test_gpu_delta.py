"""GPU parity of the delta predictor on the codes (opts.predictor = 1) against the oracle: stream bytes of nz_compress,
nz_reduce_frames and nz_reduce_local, decoded values of nz_decompress, the flags in stream and frame headers, and the
rejections (caller and stream disagree, a frame whose flag contradicts its stream)."""
import numpy as np
import pytest

import oracle
from paper_2605_12396_amd import workloads as W
from test_gpu_parity import (_first_diff, check_compress, check_decompress, gpu_compress, gpu_decompress, gpu_reduce,
                             gpu_reduce_local)

pytestmark = pytest.mark.gpu

EB1 = float(np.float32(32.0 / 63.0))          # step = 1 exactly: x = q for integers of magnitude up to 32767


@pytest.fixture(scope="module")
def nz(gpu_device):
    from paper_2605_12396_amd import binding
    binding.lib()
    return binding


def _smooth(n, seed, amp=1.0, noise=1e-4, period=300.0):
    rng = np.random.default_rng(seed)
    return (amp * np.sin(np.arange(n) / period) + noise * rng.normal(size=n)).astype(np.float32)


def _cases():
    rng = np.random.default_rng(5)
    yield "smooth_1MBframes", _smooth(1 << 20, 1), 1e-4, dict(chunk_elems=262144)
    yield "c1_field_64KBframes", W.smooth_field((256, 64, 64), seed=1), 1e-4, dict(chunk_elems=16384)
    x = W.gradient_like(1 << 20, seed=2)
    yield "gradient_1MBframes", x, W.abs_bound_from_rel(x, 1e-4), dict(chunk_elems=262144)
    yield "smooth_K1024", _smooth(300000, 2), 1e-5, dict(chunk_elems=100000, alphabet=1024)
    yield "smooth_K16", _smooth(100000, 3), 1e-4, dict(chunk_elems=30000, alphabet=16)
    yield "ragged_tail", _smooth(70001, 4), 1e-4, dict(chunk_elems=20000)
    yield "chunk_not_multiple_of_4", _smooth(30011, 5), 1e-4, dict(chunk_elems=10003)
    yield "n1", np.array([0.123], np.float32), 1e-3, dict()
    yield "tiny", _smooth(37, 6), 1e-4, dict(chunk_elems=16)
    yield "one_segment_and_a_bit", _smooth(257, 7), 1e-4, dict()
    yield "all_zero", np.zeros(50000, np.float32), 1e-4, dict(chunk_elems=16384)
    yield "constant", np.full(50000, 0.777, np.float32), 1e-4, dict(chunk_elems=16384)
    yield "uniform_noise", W.sweep_payload("uniform", 200000, 50), 1e-4, dict(chunk_elems=65536)
    # full-range codes with alternating signs: differences of up to 65534 escape, FIXEDLEN needs 17 bits
    q = rng.integers(-32767, 32768, 100000)
    yield "full_range_codes", q.astype(np.float32), EB1, dict(chunk_elems=32768)
    alt = (32767 * (1 - 2 * (np.arange(70000) & 1))).astype(np.float32)
    yield "alternating_extremes", alt, EB1, dict(chunk_elems=32768)
    y = _smooth(100000, 8)
    y[[5, 40000, 99999]] = [np.nan, np.inf, -1e30]
    yield "nan_inf_frames_raw", y, 1e-4, dict(chunk_elems=16384)
    yield "max_chunk", _smooth((1 << 20) + 5000, 9), 3e-4, dict(chunk_elems=1 << 20)
    # steps of a staircase: long runs of zero differences with rare large ones
    st = np.repeat(rng.integers(-20000, 20000, 400), 500).astype(np.float32)
    yield "staircase", st, EB1, dict(chunk_elems=65536)


@pytest.mark.parametrize("name,x,eb,kw", list(_cases()), ids=[c[0] for c in _cases()])
def test_compress_bytes_and_decompress_values_match_oracle(nz, name, x, eb, kw):
    ref, ores = check_compress(nz, x, eb, predictor=1, **kw)
    assert int(ref[36:40].view(np.uint32)[0]) == 1
    check_decompress(nz, ref, x, eb, predictor=1, **kw)


@pytest.mark.parametrize("codec", [0, 1, 2])
@pytest.mark.parametrize("kind", ["smooth", "laplace", "uniform"])
def test_pinned_codecs(nz, codec, kind):
    x = _smooth(150000, 11) if kind == "smooth" else W.sweep_payload(kind, 150000, 12)
    kw = dict(chunk_elems=40000, force_codec=codec, predictor=1)
    ref, ores = check_compress(nz, x, 1e-4, **kw)
    assert (ores.n_raw, ores.n_fixed, ores.n_huff)[codec] == ores.n_frames
    check_decompress(nz, ref, x, 1e-4, **kw)


def test_smooth_data_gets_smaller_than_without_the_predictor(nz):
    x = _smooth(1 << 20, 21)
    g1, g0 = nz.make_opts(chunk_elems=262144, predictor=1), nz.make_opts(chunk_elems=262144)
    _, r1, _ = gpu_compress(nz, x, 1e-4, g1)
    _, r0, _ = gpu_compress(nz, x, 1e-4, g0)
    assert r1["bytes"] < 0.5 * r0["bytes"]


def test_wrapping_differences_decode_to_the_oracles_codes(nz):
    """Streams made by the oracle's frame encoder from codes near +-2^30 (sums of a long reduce chain): differences
    pass 2^31 in magnitude and wrap; the receiver's running sums wrap back."""
    rng = np.random.default_rng(31)
    n = 3000
    q = (rng.integers(0, 2, n) * 2 - 1).astype(np.int64) * (2 ** 30 - rng.integers(0, 1000, n))
    o = oracle.make_opts(chunk_elems=n, predictor=1)
    g = nz.make_opts(chunk_elems=n, predictor=1)
    from crafted import single_frame_stream
    step_bits = int(oracle.step_constants(EB1)[0].view(np.uint32))
    for codec in (1, 2):
        fr = oracle.frame_encode(q.astype(np.int32), codec, o, step_bits=step_bits)
        s = single_frame_stream(n, n, step_bits, fr.tobytes())
        s[36:40] = np.array([1], np.uint32).view(np.uint8)
        ref, ores, orc = oracle.decompress(s, n, EB1)
        assert orc == 0
        rc, r, got = gpu_decompress(nz, s, n, EB1, g)
        assert rc == 0 and r["status"] == 0
        assert (got.view(np.uint32) == ref.view(np.uint32)).all()
        assert (got == q.astype(np.float32)).all()


def test_predictor_flags_are_checked(nz):
    x = _smooth(100000, 41)
    kw = dict(chunk_elems=32768)
    g1, g0 = nz.make_opts(predictor=1, **kw), nz.make_opts(**kw)
    s1, _, _ = oracle.compress(x, 1e-4, oracle.make_opts(predictor=1, **kw))
    s0, _, _ = oracle.compress(x, 1e-4, oracle.make_opts(**kw))
    # the caller and the stream disagree: told so, nothing written
    for s, g in ((s1, g0), (s0, g1)):
        rc, r, got = gpu_decompress(nz, s, x.size, 1e-4, g)
        assert r["status"] == nz.ERR_MISMATCH and (got == 7.0).all()
    # a stream header with an unknown predictor is corrupt
    bad = s1.copy(); bad[36] = 2
    _, ores, orc = oracle.decompress(bad, x.size, 1e-4)
    rc, r, got = gpu_decompress(nz, bad, x.size, 1e-4, g1)
    assert orc == nz.ERR_CORRUPT and r["status"] == nz.ERR_CORRUPT and (got == 7.0).all()
    # a frame whose flag contradicts the stream's (check word made consistent): that frame is rejected and zero-filled
    for s, g, flag in ((s1, g1, 0), (s0, g0, 1)):
        bad = s.copy()
        off = int(bad[64 + 8:64 + 16].view(np.uint64)[0])             # frame 1
        h = bad[off:off + 32].view(np.uint32).copy()
        assert h[1] in (1, 2)
        h[5] = (h[5] & 0x7FFFFFFF) | (flag << 31)
        h[7] = 0x5A5A5A5A ^ h[0] ^ h[1] ^ h[2] ^ h[3] ^ h[4] ^ h[5] ^ h[6]
        bad[off:off + 32] = h.view(np.uint8)
        ref, ores, orc = oracle.decompress(bad, x.size, 1e-4)
        rc, r, got = gpu_decompress(nz, bad, x.size, 1e-4, g)
        assert orc == nz.ERR_CORRUPT and r["status"] == nz.ERR_CORRUPT
        assert (got.view(np.uint32) == ref.view(np.uint32)).all() and (got[32768:65536] == 0).all()
    # the sampled and the stochastic paths are not built with the predictor
    import torch
    sess = nz.Session(x.size, g1, "cuda:0", reduce=True)
    out = sess.new_stream_buffer()
    dx = torch.from_numpy(x).to("cuda:0")
    assert nz.nz_compress_sr(dx, x.size, 1e-4, 1, out, sess.cap, sess.res, g1, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_workspace_bytes(x.size, nz.make_opts(predictor=2)) == 0
    assert nz.nz_workspace_bytes(x.size, nz.make_opts(reserved=1)) == 0
    torch.cuda.synchronize()


def _reduce_case(nz, a, b, eb, **kw):
    g, o = nz.make_opts(predictor=1, **kw), oracle.make_opts(predictor=1, **kw)
    sa, _, rca = oracle.compress(a, eb, o)
    sb, _, rcb = oracle.compress(b, eb, o)
    ref, ores, orc = oracle.reduce_frames(sa, sb, a.size, eb, o)
    rc, r, got = gpu_reduce(nz, sa, sb, a.size, eb, g)
    assert rca == 0 and rcb == 0 and orc == 0 and rc == 0 and r["status"] == 0
    assert (r["n_raw"], r["n_fixed"], r["n_huff"], r["bytes"]) == (ores.n_raw, ores.n_fixed, ores.n_huff, ores.bytes)
    assert _first_diff(got, ref) == -1, "first differing byte at %d" % _first_diff(got, ref)
    return sa, sb, ref


@pytest.mark.parametrize("name", ["smooth", "gradient", "ragged", "wide_sums", "raw_operand", "fixed_operands", "big_frames"])
def test_reduce_frames_matches_oracle(nz, name):
    if name == "smooth":
        _reduce_case(nz, _smooth(300000, 51), _smooth(300000, 52, amp=0.7, period=170.0), 1e-4, chunk_elems=65536)
    elif name == "gradient":
        a, b = W.gradient_like(300000, seed=53), W.gradient_like(300000, seed=54)
        _reduce_case(nz, a, b, 1e-5, chunk_elems=100000)
    elif name == "ragged":
        _reduce_case(nz, _smooth(70001, 55), _smooth(70001, 56, amp=0.5), 1e-4, chunk_elems=20000)
    elif name == "wide_sums":
        # sums of magnitude up to 65534 need the 32-bit side array; their differences reach 131068
        rng = np.random.default_rng(57)
        a = (32767 * (1 - 2 * (np.arange(200000) & 1))).astype(np.float32)
        b = a.copy(); b[rng.integers(0, 200000, 5000)] *= -1
        _reduce_case(nz, a, b, EB1, chunk_elems=65536)
    elif name == "raw_operand":
        a = _smooth(100000, 58); a[40000] = np.nan
        _reduce_case(nz, a, _smooth(100000, 59), 1e-4, chunk_elems=16384)
    elif name == "fixed_operands":
        a, b = W.sweep_payload("uniform", 200000, 60), W.sweep_payload("uniform", 200000, 61)
        _reduce_case(nz, a, b, 1e-4, chunk_elems=65536)
    else:
        _reduce_case(nz, _smooth((1 << 20) + 777, 62), _smooth((1 << 20) + 777, 63, amp=0.3), 1e-4, chunk_elems=1 << 19)


def test_reduce_chain_and_local_step(nz):
    """A four-rank chain: the reduce of delta-coded streams equals the delta-coded stream of the summed codes, and the
    fused ring step (incoming stream + own fp32 data) gives the same bytes as compressing and reducing."""
    n = 250000
    kw = dict(chunk_elems=65536)
    g, o = nz.make_opts(predictor=1, **kw), oracle.make_opts(predictor=1, **kw)
    xs = [_smooth(n, 70 + i, amp=0.5 + 0.1 * i, period=200.0 + 30 * i) for i in range(4)]
    eb = 1e-4
    acc, _, _ = oracle.compress(xs[0], eb, o)
    for x in xs[1:]:
        ref, ores, orc = oracle.reduce_local(acc, x, eb, o)
        rc, r, got = gpu_reduce_local(nz, acc, x, eb, g)
        assert orc == 0 and rc == 0 and r["status"] == 0 and r["bytes"] == ores.bytes
        assert _first_diff(got, ref) == -1
        sx, _, _ = oracle.compress(x, eb, o)
        two, _, _ = oracle.reduce_frames(acc, sx, n, eb, o)
        assert (two == ref).all()
        acc = ref
    rc, r, got = gpu_decompress(nz, acc, n, eb, g)
    want, _, _ = oracle.decompress(acc, n, eb)
    assert r["status"] == 0 and (got.view(np.uint32) == want.view(np.uint32)).all()
    assert np.abs(got.astype(np.float64) - np.sum(np.stack(xs).astype(np.float64), 0)).max() <= 4 * eb * (1 + 1e-6) + 1e-6


def test_reduce_local_frame_kinds_and_mismatch(nz):
    n = 100000
    kw = dict(chunk_elems=16384)
    g, o = nz.make_opts(predictor=1, **kw), oracle.make_opts(predictor=1, **kw)
    a = _smooth(n, 81); a[20000] = np.inf                       # an incoming RAW frame
    x = _smooth(n, 82); x[70000] = 1e30                         # local data that cannot be quantized
    sa, _, _ = oracle.compress(a, 1e-4, o)
    ref, ores, orc = oracle.reduce_local(sa, x, 1e-4, o)
    rc, r, got = gpu_reduce_local(nz, sa, x, 1e-4, g)
    assert orc == 0 and rc == 0 and r["status"] == 0 and r["n_raw"] == ores.n_raw >= 2
    assert _first_diff(got, ref) == -1
    # operands made without the predictor are refused by a caller that asks for it, and the other way round
    s0, _, _ = oracle.compress(_smooth(n, 83), 1e-4, oracle.make_opts(**kw))
    rc, r, got = gpu_reduce_local(nz, s0, x, 1e-4, g)
    assert r["status"] == nz.ERR_MISMATCH
    rc, r, got = gpu_reduce(nz, sa, s0, n, 1e-4, g)
    assert r["status"] == nz.ERR_MISMATCH
    rc, r, got = gpu_reduce(nz, sa, sa, n, 1e-4, nz.make_opts(**kw))
    assert r["status"] == nz.ERR_MISMATCH


@pytest.mark.parametrize("seed", range(10))
def test_seeded_sweep(nz, seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 400000))
    chunk = int(rng.choice([16, 1000, 4096, 10003, 65536, 262144]))
    K = int(rng.choice([16, 64, 256, 1024]))
    eb = float(10.0 ** rng.uniform(-5, -2))
    kind = seed % 3
    x = _smooth(n, seed, amp=float(rng.uniform(0.1, 3)), noise=float(10.0 ** rng.uniform(-5, -2)), period=float(rng.uniform(20, 2000)))
    if kind == 1:
        x = W.gradient_like(n, seed=seed)
    if kind == 2 and n > 10:
        x[rng.integers(0, n, 3)] = [np.nan, 1e20, -np.inf]
    kw = dict(chunk_elems=chunk, alphabet=K, predictor=1)
    ref, _ = check_compress(nz, x, eb, **kw)
    check_decompress(nz, ref, x, eb, **kw)
    y = _smooth(n, seed + 100, amp=0.3)
    sy, _, _ = oracle.compress(y, eb, oracle.make_opts(**kw))
    red, ores, orc = oracle.reduce_frames(ref, sy, n, eb, oracle.make_opts(**kw))
    rc, r, got = gpu_reduce(nz, ref, sy, n, eb, nz.make_opts(**kw))
    assert orc == 0 and rc == 0 and r["status"] == 0 and _first_diff(got, red) == -1


def test_full_size_message_with_the_predictor(nz):
    """A 64 Mi-element message in 1 MiB frames (the headline geometry) with the predictor on: a smooth signal plus
    gradient-like noise, compressed stream, decompressed values and the ring-step reduce against the oracle."""
    import torch
    n = 1 << 26
    noise = W.gradient_like(n, seed=5)
    x = (np.sin(np.arange(n, dtype=np.float64) / 700.0) + noise).astype(np.float32)
    eb = float(np.float32(W.abs_bound_from_rel(x, 1e-4)))
    kw = dict(chunk_elems=262144, predictor=1)
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
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
    rc, red = sess.reduce_local(out, nbytes, torch.from_numpy(noise).to("cuda:0"), n, eb)
    rr = sess.result()
    ro, rres, rrc = oracle.reduce_local(ref, noise, eb, o)
    assert rc == 0 and rrc == 0 and rr["status"] == 0 and rr["bytes"] == rres.bytes
    assert _first_diff(red[:rr["bytes"]].cpu().numpy(), ro) == -1


@pytest.mark.parametrize("predictor", [1, 0], ids=["delta", "plain"])
def test_garbage_in_streams_with_fixedlen_and_huffman_frames(nz, predictor):
    """Byte flips anywhere behind the stream header of a stream that holds HUFFMAN, FIXEDLEN and RAW frames: never a
    fault, the oracle's verdict, and the oracle's output in every element (FIXEDLEN and RAW payloads cannot be told
    from valid ones: their garbage decodes to the same values on both sides; with the predictor a flipped difference
    moves the rest of its segment)."""
    n = 5 * 16384 + 777
    x = np.concatenate([W.gradient_like(2 * 16384, seed=91), W.sweep_payload("uniform", 2 * 16384, 92),
                        W.gradient_like(16384 + 777, seed=93)])
    x[3 * 16384 + 5] = np.inf                                           # frame 3 is RAW
    eb = 1e-4
    kw = dict(chunk_elems=16384, predictor=predictor)
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    s, sres, rc = oracle.compress(x, eb, o)
    assert rc == 0 and sres.n_raw == 1 and sres.n_fixed >= 1 and sres.n_huff >= 2
    rng = np.random.default_rng(17 + predictor)
    base = 64 + 8 * 6
    n_rejected = 0
    for trial in range(80):
        t = s.copy()
        for _ in range(int(rng.integers(1, 4))):
            t[int(rng.integers(base, s.size))] ^= int(rng.integers(1, 256))
        oref, ores, orc = oracle.decompress(t, n, eb)
        rc, r, got = gpu_decompress(nz, t, n, eb, g)
        assert r["status"] == orc, (trial, r, orc)
        if orc in (0, nz.ERR_CORRUPT) and ores.bytes:
            assert (r["n_raw"], r["n_fixed"], r["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff), trial
            assert (got.view(np.uint32) == oref.view(np.uint32)).all(), trial
        n_rejected += orc != 0
        if trial % 4 == 0:                                               # the same stream through the ring step
            ored, rres, rrc = oracle.reduce_local(t, x, eb, o)
            rc2, r2, got2 = gpu_reduce_local(nz, t, x, eb, g)
            assert r2["status"] == rrc, (trial, r2, rrc)
            if rrc == 0:
                assert r2["bytes"] == rres.bytes and _first_diff(got2, ored) == -1, trial
    assert n_rejected > 10
