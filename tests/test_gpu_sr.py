"""GPU parity of the stochastic interface quantizer (nz_compress_sr, nz_qsgd_step, the *_step receivers) against the
oracle: identical draws, codes, selector decisions and stream bytes; decoded values; exact integer reduce."""
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


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def gpu_compress_sr(nz, x, step, seed, g):
    sess = nz.Session(x.size, g, "cuda:0", reduce=True)
    out = sess.new_stream_buffer()
    rc = nz.nz_compress_sr(_dev(x), x.size, step, seed, out, sess.cap, sess.res, g, sess.ws, sess.ws_bytes)
    r = sess.result()
    return rc, r, out, sess


def check_sr(nz, x, step, seed, **kw):
    import torch
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    ref, ores, orc = oracle.compress_sr(x, step, seed, o)
    rc, r, out, sess = gpu_compress_sr(nz, x, step, seed, g)
    assert rc == 0 and orc == 0 and r["status"] == 0
    assert (r["n_raw"], r["n_fixed"], r["n_huff"], r["bytes"]) == (ores.n_raw, ores.n_fixed, ores.n_huff, ores.bytes)
    got = out[:r["bytes"]].cpu().numpy()
    d = np.nonzero(got != ref)[0]
    assert d.size == 0, "first differing byte %d" % int(d[0])
    y = torch.full((x.size,), 7.0, dtype=torch.float32, device="cuda:0")
    assert nz.nz_decompress_step(out, r["bytes"], y, x.size, step, sess.res, g, sess.ws, sess.ws_bytes) == 0
    assert sess.result()["status"] == 0
    yo, _, drc = oracle.decompress_step(ref, x.size, step)
    y = y.cpu().numpy()
    assert drc == 0 and (y.view(np.uint32) == yo.view(np.uint32)).all()
    fin = np.isfinite(x)
    assert (np.abs(y[fin].astype(np.float64) - x[fin]) <= float(np.float32(step)) * (1 + 2.0 ** -6)).all()
    return ref, out, r, sess


def _cases():
    rng = np.random.default_rng(17)
    x = W.gradient_like(1 << 20, seed=2)
    yield "gradient_1MBframes_s256", x, oracle.qsgd_step(x, 256), 1, dict(chunk_elems=262144)
    yield "gradient_s4", x[:300000], oracle.qsgd_step(x[:300000], 4), 2, dict(chunk_elems=65536)
    yield "gradient_s32767_K1024", x[:200000], oracle.qsgd_step(x[:200000], 32767), 3, dict(chunk_elems=100000, alphabet=1024)
    yield "ragged_chunk_not_multiple_of_4", W.gradient_like(30011, seed=5), 3e-4, 4, dict(chunk_elems=10003)
    yield "n1", np.array([0.123], np.float32), 0.05, 5, dict()
    yield "tiny", W.gradient_like(37, seed=6), 1e-4, 6, dict(chunk_elems=16)
    yield "uniform_fixedlen", W.sweep_payload("uniform", 200000, 50), 1e-4, 7, dict(chunk_elems=65536)
    yield "all_zero", np.zeros(50000, np.float32), 1e-4, 8, dict(chunk_elems=16384)
    yield "grid_points", (rng.integers(-300, 300, 100000) * 0.25).astype(np.float32), 0.25, 9, dict(chunk_elems=32768)
    y = W.gradient_like(100000, seed=8)
    y[[5, 40000, 99999]] = [np.nan, np.inf, -1e30]
    yield "nan_inf_frames_raw", y, 1e-4, 10, dict(chunk_elems=16384)
    yield "pinned_huffman", W.gradient_like(150000, seed=9), 2e-4, 11, dict(chunk_elems=40000, force_codec=2)
    yield "pinned_fixedlen", W.gradient_like(150000, seed=9), 2e-4, 12, dict(chunk_elems=40000, force_codec=1)
    yield "max_chunk", W.gradient_like((1 << 20) + 5000, seed=7), 3e-4, 13, dict(chunk_elems=1 << 20)
    yield "seed_high_bits", W.gradient_like(70001, seed=4), 1e-4, 0xFFFFFFFF, dict(chunk_elems=20000)


@pytest.mark.parametrize("name,x,step,seed,kw", list(_cases()), ids=[c[0] for c in _cases()])
def test_sr_stream_and_values_match_oracle(nz, name, x, step, seed, kw):
    check_sr(nz, x, float(np.float32(step)), seed, **kw)


def test_qsgd_step_and_reduce(nz):
    import torch
    n = 300000
    kw = dict(chunk_elems=65536)
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    a, b = W.gradient_like(n, seed=40), W.gradient_like(n, seed=41)
    ws = torch.empty(8192, dtype=torch.uint8, device="cuda:0")
    st = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    for x, levels in ((a, 256), (b, 16), (a, 32767), (np.zeros(100, np.float32), 8)):
        assert nz.nz_qsgd_step(_dev(x), x.size, levels, st, ws, 8192) == 0
        got, ref = float(st.cpu()[0]), oracle.qsgd_step(x, levels)
        assert abs(got - ref) <= 2.0 ** -23 * ref                       # within one unit in the last place
    assert nz.nz_qsgd_step(_dev(a), n, 0, st, ws, 8192) == nz.ERR_INVALID
    assert nz.nz_qsgd_step(_dev(a), n, 40000, st, ws, 8192) == nz.ERR_INVALID
    # the two ranks agree on the larger width, compress with their own seeds, and the reduce adds the codes exactly
    step = float(np.float32(max(oracle.qsgd_step(a, 256), oracle.qsgd_step(b, 256))))
    ref_a, out_a, r_a, sess = check_sr(nz, a, step, 5, **kw)
    ref_b, out_b, r_b, _ = check_sr(nz, b, step, 6, **kw)
    red, rres, rrc = oracle.reduce_frames_step(ref_a, ref_b, n, step, o)
    out = sess.new_stream_buffer()
    rc = nz.nz_reduce_frames_step(out_a, r_a["bytes"], out_b, r_b["bytes"], out, sess.cap, n, step, sess.res, g, sess.ws, sess.ws_bytes)
    r = sess.result()
    assert rc == 0 and rrc == 0 and r["status"] == 0 and r["bytes"] == rres.bytes
    assert (out[:r["bytes"]].cpu().numpy() == red).all()
    # a receiver with another width is told so
    y = torch.empty(n, dtype=torch.float32, device="cuda:0")
    nz.nz_decompress_step(out_a, r_a["bytes"], y, n, step * 2, sess.res, g, sess.ws, sess.ws_bytes)
    assert sess.result()["status"] == nz.ERR_MISMATCH
    assert nz.nz_compress_sr(_dev(a), n, 0.0, 1, out, sess.cap, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_compress_sr(_dev(a), n, float("nan"), 1, out, sess.cap, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    torch.cuda.synchronize()


def test_sr_index_past_32_bits(nz):
    """Draws are keyed by the 64-bit message index: a message longer than 2^32 elements, checked on its last frames
    (which lie beyond the wrap of the low half) against the oracle's quantizer run with the same first index."""
    import torch
    n = (1 << 32) + 3 * 65536 + 777
    chunk = 1 << 20
    g = nz.make_opts(chunk_elems=chunk)
    x = torch.empty(n, dtype=torch.float32, device="cuda:0")
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(11)
    x.normal_(0.0, 1e-3, generator=gen)
    step, seed = 1e-4, 77
    sess = nz.Session(n, g, "cuda:0")
    out = sess.new_stream_buffer()
    assert nz.nz_compress_sr(x, n, step, seed, out, sess.cap, sess.res, g, sess.ws, sess.ws_bytes) == 0
    r = sess.result()
    nfr = (n + chunk - 1) // chunk
    assert r["status"] == 0 and r["n_frames"] == nfr
    offs = out[64:64 + 8 * nfr].cpu().numpy().view(np.uint64).astype(np.int64)
    o = oracle.make_opts(chunk_elems=chunk)
    step_bits = int(np.float32(step).view(np.uint32))
    for k in (nfr - 1, nfr - 2, 4095):                       # frame 4095 ends at the wrap, frame 4096 starts on it
        i0 = k * chunk
        xf = x[i0:min(n, i0 + chunk)].cpu().numpy()
        q, ok = oracle.sr_quantize(xf, step, seed, first_index=i0)
        assert ok.all()
        plan = oracle.frame_plan(q, o)
        fr = oracle.frame_encode(q, plan["codec"], o, step_bits=step_bits)
        got = out[int(offs[k]):int(offs[k]) + fr.size].cpu().numpy()
        assert (got == fr).all(), k


def _gpu_reduce_local_sr(nz, a_stream, x, step, seed, g):
    import torch
    n = x.size
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    da = _dev(np.concatenate([a_stream, np.zeros((-a_stream.size) % 16, np.uint8)]))
    out = sess.new_stream_buffer()
    rc = nz.nz_reduce_local_sr(da, a_stream.size, _dev(x), out, sess.cap, n, step, seed, sess.res, g, sess.ws, sess.ws_bytes)
    r = sess.result()
    return rc, r, out[:r["bytes"]].cpu().numpy()


@pytest.mark.parametrize("name", ["ring_chain", "ragged_small_frames", "raw_and_unquantizable", "big_frames", "fixedlen_in"])
def test_ring_step_with_the_stochastic_quantizer(nz, name):
    """nz_reduce_local_sr against the oracle: bytes of every step of a chain, frames that turn RAW, large frames on the
    vectorised path, and the refusals."""
    if name == "ring_chain":
        n, kw, peers = 300000, dict(chunk_elems=65536), 4
    elif name == "ragged_small_frames":
        n, kw, peers = 30011, dict(chunk_elems=10003), 3
    elif name == "big_frames":
        n, kw, peers = 2 * 262144 + 70001, dict(chunk_elems=262144), 3
    else:
        n, kw, peers = 100000, dict(chunk_elems=16384), 2
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    xs = [W.gradient_like(n, seed=200 + p) for p in range(peers)]
    if name == "fixedlen_in":
        xs[0] = W.sweep_payload("uniform", n, 77)
    step = float(np.float32(max(oracle.qsgd_step(x, 200) for x in xs)))
    if name == "raw_and_unquantizable":
        xs[0][5] = np.inf                                   # incoming RAW frame
        xs[1][40000] = np.nan                               # local value that cannot be quantized
        xs[1][70000] = np.float32(40000.0 * step)           # beyond 32767 bins
    acc, _, rc = oracle.compress_sr(xs[0], step, 100, o)
    assert rc == 0
    for p in range(1, peers):
        ref, ores, orc = oracle.reduce_local_sr(acc, xs[p], step, 100 + p, o)
        rc, r, got = _gpu_reduce_local_sr(nz, acc, xs[p], step, 100 + p, g)
        assert orc == 0 and rc == 0 and r["status"] == 0, (p, r)
        assert (r["n_raw"], r["n_fixed"], r["n_huff"], r["bytes"]) == (ores.n_raw, ores.n_fixed, ores.n_huff, ores.bytes)
        d = np.nonzero(got != ref)[0]
        assert d.size == 0, "step %d: first differing byte %d" % (p, int(d[0]))
        acc = ref
    if name == "raw_and_unquantizable":
        assert ores.n_raw == 3
    if name == "ring_chain":
        import torch
        sess = nz.Session(n, g, "cuda:0", reduce=True)
        da = _dev(np.concatenate([acc, np.zeros((-acc.size) % 16, np.uint8)]))
        out = sess.new_stream_buffer()
        dx = _dev(xs[1])
        # a stream made with another width, a predictor, a bad width
        assert nz.nz_reduce_local_sr(da, acc.size, dx, out, sess.cap, n, step * 2, 1, sess.res, g, sess.ws, sess.ws_bytes) == 0
        assert sess.result()["status"] == nz.ERR_MISMATCH
        gp = nz.make_opts(predictor=1, **kw)
        assert nz.nz_reduce_local_sr(da, acc.size, dx, out, sess.cap, n, step, 1, sess.res, gp, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
        assert nz.nz_reduce_local_sr(da, acc.size, dx, out, sess.cap, n, float("nan"), 1, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
        torch.cuda.synchronize()


@pytest.mark.parametrize("kw", [dict(force_codec=0), dict(min_gain_permil=999)])
def test_ring_step_sums_committed_raw_with_the_stochastic_quantizer(nz, kw):
    """A frame of integer sums that the selector commits RAW holds the fp32 sums of the dequantized operands; the
    stochastic ring step recovers the rank's own codes with the same draws."""
    n, chunk = 150001, 65536
    g, o = nz.make_opts(chunk_elems=chunk, **kw), oracle.make_opts(chunk_elems=chunk, **kw)
    xs = [W.gradient_like(n, seed=230 + p) for p in range(2)]
    step = float(np.float32(max(oracle.qsgd_step(x, 200) for x in xs)))
    acc, _, rc = oracle.compress_sr(xs[0], step, 7, oracle.make_opts(chunk_elems=chunk))
    assert rc == 0
    ref, ores, orc = oracle.reduce_local_sr(acc, xs[1], step, 8, o)
    rc, r, got = _gpu_reduce_local_sr(nz, acc, xs[1], step, 8, g)
    assert orc == 0 and rc == 0 and r["status"] == 0 and ores.n_raw == 3
    assert (r["n_raw"], r["bytes"]) == (ores.n_raw, ores.bytes)
    d = np.nonzero(got != ref)[0]
    assert d.size == 0, "first differing byte %d" % int(d[0])
