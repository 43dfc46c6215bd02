"""GPU parity of the k-ary reduce (nz_reduce_k through the C ABI) against the CPU oracle: output streams byte for
byte over operand counts, codecs, alphabets, the predictor, ragged frames, wide codes, RAW operands in any position,
partial sums that leave the integer range at an operand in the middle, gates, refusals."""
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


def gpu_reduce_k(nz, streams, n, eb, g, cap=None):
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    ds = [_dev(np.concatenate([s, np.zeros((-s.size) % 16, np.uint8)])) for s in streams]
    rc, out = sess.reduce_k(ds, [s.size for s in streams], n, eb, cap=cap)
    r = sess.result()
    return rc, r, out[:r["bytes"]].cpu().numpy()


def check(nz, streams, n, eb, **kw):
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    ref, ores, orc = oracle.reduce_k(streams, n, eb, o)
    rc, r, got = gpu_reduce_k(nz, streams, n, eb, g)
    assert orc == 0 and rc == 0 and r["status"] == 0, (orc, rc, r)
    assert (r["n_raw"], r["n_fixed"], r["n_huff"], r["n_frames"]) == (ores.n_raw, ores.n_fixed, ores.n_huff, ores.n_frames)
    assert r["bytes"] == ores.bytes
    d = np.nonzero(got != ref)[0]
    assert d.size == 0, "first differing byte %d" % int(d[0])
    return ref, ores


@pytest.mark.parametrize("k", [2, 3, 4, 7, 8])
@pytest.mark.parametrize("n,chunk", [(300000, 65536), (2 * 262144 + 70001, 262144), (30011, 10003)])
def test_matches_the_oracle(nz, k, n, chunk):
    eb = 1e-4
    o = oracle.make_opts(chunk_elems=chunk)
    xs = [W.gradient_like(n, seed=400 + p, b=1e-3 * (1 + p % 3)) for p in range(k)]
    ss = [oracle.compress(x, eb, o)[0] for x in xs]
    ref, ores = check(nz, ss, n, eb, chunk_elems=chunk)
    # (the oracle's result is the chain of two-operand reduces)
    acc = ss[0]
    for s in ss[1:]:
        acc = oracle.reduce_frames(acc, s, n, eb, o)[0]
    assert np.array_equal(acc, ref)


@pytest.mark.parametrize("kw", [dict(alphabet=1024), dict(predictor=1), dict(force_codec=1), dict(force_codec=2), dict(alphabet=16),
                                dict(force_codec=0), dict(min_gain_permil=700), dict(predictor=1, force_codec=1)])
def test_options(nz, kw):
    n, eb, chunk, k = 200000, 1e-4, 65536, 5
    src = {kk: v for kk, v in kw.items() if kk in ("alphabet", "predictor")}
    o = oracle.make_opts(chunk_elems=chunk, **src)
    xs = [W.gradient_like(n, seed=420 + p) for p in range(k)]
    ss = [oracle.compress(x, eb, o)[0] for x in xs]
    check(nz, ss, n, eb, chunk_elems=chunk, **kw)


def test_operand_codecs_mixed(nz):
    # operands coded RAW / FIXEDLEN / HUFFMAN in turn, dense and sparse payloads
    n, eb, chunk = 150001, 1e-4, 40000
    xs = [W.gradient_like(n, seed=430), W.sweep_payload("uniform", n, 431), W.gradient_like(n, seed=432, b=3e-2),
          W.sweep_payload("sinusoid", n, 433), np.zeros(n, np.float32), W.gradient_like(n, seed=435)]
    forces = [2, 1, -1, 0, -1, 1]
    ss = [oracle.compress(x, eb, oracle.make_opts(chunk_elems=chunk, force_codec=f))[0] for x, f in zip(xs, forces)]
    for order in ([0, 1, 2, 3, 4, 5], [3, 0, 1, 2, 4, 5], [0, 1, 2, 4, 5, 3], [5, 4, 3, 2, 1, 0]):
        check(nz, [ss[i] for i in order], n, eb, chunk_elems=chunk)


def test_wide_codes_raw_operands_and_nan(nz):
    n, eb, chunk = 4 * 65536 + 100, 1e-3, 65536
    o = oracle.make_opts(chunk_elems=chunk)
    xs = [W.gradient_like(n, seed=440 + p) for p in range(5)]
    xs[0][7] = 30.0; xs[1][7] = 31.0; xs[2][65536 + 9] = -25.0          # codes and sums beyond 16 bits in the staging
    xs[2][2 * 65536 + 5] = np.nan                                       # frame 2 RAW from operand 2 on
    xs[0][3 * 65536 + 1] = np.inf; xs[4][3 * 65536 + 2] = -np.inf       # frame 3 RAW from the start, NaN sum at the end? (inf + -inf elsewhere)
    xs[4][3 * 65536 + 1] = -np.inf                                      # inf + (-inf) = NaN, stored as the canonical NaN
    ss = [oracle.compress(x, eb, o)[0] for x in xs]
    ref, ores = check(nz, ss, n, eb, chunk_elems=chunk)
    assert ores.n_raw == 2
    for order in ([2, 0, 1, 3, 4], [0, 1, 3, 4, 2], [4, 3, 2, 1, 0]):
        check(nz, [ss[i] for i in order], n, eb, chunk_elems=chunk)


def test_partial_sum_leaves_the_range_in_the_middle(nz):
    n, eb, chunk = 2 * 65536 + 500, 1e-3, 65536
    o = oracle.make_opts(chunk_elems=chunk)
    step, _ = oracle.step_constants(eb)
    y = (W.gradient_like(n, seed=450) * 0).astype(np.float32)
    y[3] = step; y[4] = -step; y[70000] = step
    t = oracle.compress(y, eb, o)[0]
    for _ in range(29):
        t = oracle.reduce_frames(t, t, n, eb, o)[0]                      # codes +-2^29
    small = oracle.compress(W.gradient_like(n, seed=451), eb, o)[0]
    z = oracle.compress(np.zeros(n, np.float32), eb, o)[0]
    ref, ores = check(nz, [t, t, z, small], n, eb, chunk_elems=chunk)    # 2^30 exactly, then small codes: range flag by the slow path
    for ops in ([t, t, small, t], [small, t, t, t], [t, small, t, t, z], [t, t, t], [z, t, t, t, small, small]):
        ref, ores = check(nz, ops, n, eb, chunk_elems=chunk)
        assert ores.n_raw >= 1


def test_refusals(nz):
    import torch
    n, eb, chunk = 100000, 1e-4, 16384
    g, o = nz.make_opts(chunk_elems=chunk), oracle.make_opts(chunk_elems=chunk)
    xs = [W.gradient_like(n, seed=460 + p) for p in range(3)]
    ss = [oracle.compress(x, eb, o)[0] for x in xs]
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    ds = [_dev(np.concatenate([s, np.zeros((-s.size) % 16, np.uint8)])) for s in ss]
    sizes = [s.size for s in ss]
    out = sess.new_stream_buffer()
    assert nz.nz_reduce_k(ds[:1], sizes[:1], out, sess.cap, n, eb, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_reduce_k([ds[0]] * 65, [sizes[0]] * 65, out, sess.cap, n, eb, sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    assert nz.nz_reduce_k(ds, sizes, out, sess.cap, n, eb, sess.res, g, sess.ws, 1024) == nz.ERR_INVALID
    assert nz.nz_reduce_k(ds, sizes, out, sess.cap, n, float("nan"), sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID
    # an operand made with another bound / frame size / length: mismatch, wherever it stands; nothing is published
    bad = [oracle.compress(xs[1], 2e-4, o)[0], oracle.compress(xs[1], eb, oracle.make_opts(chunk_elems=8192))[0],
           oracle.compress(xs[1][:n - 1], eb, o)[0]]
    for b in bad:
        for pos in range(3):
            ops = list(ss); ops[pos] = b
            ref, ores, orc = oracle.reduce_k(ops, n, eb, o)
            rc, r, got = gpu_reduce_k(nz, ops, n, eb, g)
            assert orc == oracle.ERR_MISMATCH and rc == 0 and r["status"] == nz.ERR_MISMATCH and r["bytes"] == 0
    # a damaged frame in any operand: corrupt
    for pos in range(3):
        b = ss[pos].copy()
        off = int(b[64 + 8:64 + 16].view(np.uint64)[0])
        b[off + 28] ^= 0x10
        ops = list(ss); ops[pos] = b
        ref, ores, orc = oracle.reduce_k(ops, n, eb, o)
        rc, r, got = gpu_reduce_k(nz, ops, n, eb, g)
        assert orc == oracle.ERR_CORRUPT and rc == 0 and r["status"] == nz.ERR_CORRUPT and r["bytes"] == 0
    # capacity one byte short
    ref, ores, orc = oracle.reduce_k(ss, n, eb, o)
    rc, r, got = gpu_reduce_k(nz, ss, n, eb, g, cap=ref.size - 1)
    assert r["status"] == nz.ERR_CAPACITY and r["bytes"] == 0
    rc, r, got = gpu_reduce_k(nz, ss, n, eb, g, cap=ref.size)
    assert r["status"] == 0 and np.array_equal(got, ref)
    # 64 operands (the maximum)
    rc, r, got = gpu_reduce_k(nz, [ss[p % 3] for p in range(64)], n, eb, g)
    ref, ores, orc = oracle.reduce_k([ss[p % 3] for p in range(64)], n, eb, o)
    assert rc == 0 and orc == 0 and r["status"] == 0 and np.array_equal(got, ref)
    torch.cuda.synchronize()


def test_c4_full_size(nz):
    """Config 4 as bench.py runs it: eight peers of 32 Mi elements (eb = 1e-5, 1 MiB frames) reduced at once; the
    GPU compresses the peers (compress parity at this shape is covered elsewhere, and checked here for the first
    peer), the oracle reduces the same eight streams, whole message."""
    import torch
    n, eb, peers = 1 << 25, 1e-5, 8
    g, o = nz.make_opts(chunk_elems=262144), oracle.make_opts(chunk_elems=262144)
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    host, dev, sizes = [], [], []
    for p in range(peers):
        x = W.gradient_like(n, seed=40 + p, outlier_frac=0.0)
        rc, out = sess.compress(torch.from_numpy(x).to("cuda:0"), eb)
        r = sess.result()
        assert rc == 0 and r["status"] == 0
        s = out[:r["bytes"]].cpu().numpy()
        if p == 0:
            assert np.array_equal(s, oracle.compress(x, eb, o)[0])
        host.append(s); dev.append(out); sizes.append(r["bytes"])
        del x
    rc, red = sess.reduce_k(dev, sizes, n, eb)
    rr = sess.result()
    ref, ores, orc = oracle.reduce_k(host, n, eb, o)
    assert rc == 0 and orc == 0 and rr["status"] == 0 and rr["bytes"] == ores.bytes
    assert (rr["n_raw"], rr["n_fixed"], rr["n_huff"]) == (ores.n_raw, ores.n_fixed, ores.n_huff)
    got = red[:rr["bytes"]].cpu().numpy()
    d = np.nonzero(got != ref)[0]
    assert d.size == 0, "first differing byte %d" % int(d[0])


def test_streams_of_the_stochastic_quantizer(nz):
    n, chunk = 200000, 65536
    g, o = nz.make_opts(chunk_elems=chunk), oracle.make_opts(chunk_elems=chunk)
    xs = [W.gradient_like(n, seed=470 + p) for p in range(5)]
    step = float(np.float32(max(oracle.qsgd_step(x, 200) for x in xs)))
    ss = [oracle.compress_sr(x, step, 20 + p, o)[0] for p, x in enumerate(xs)]
    ref, ores, orc = oracle.reduce_k(ss, n, None, o, step=step)
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    ds = [_dev(np.concatenate([s, np.zeros((-s.size) % 16, np.uint8)])) for s in ss]
    out = sess.new_stream_buffer()
    rc = nz.nz_reduce_k_step(ds, [s.size for s in ss], out, sess.cap, n, step, sess.res, g, sess.ws, sess.ws_bytes)
    r = sess.result()
    assert rc == 0 and orc == 0 and r["status"] == 0 and r["bytes"] == ores.bytes
    assert np.array_equal(out[:r["bytes"]].cpu().numpy(), ref)
    assert nz.nz_reduce_k_step(ds, [s.size for s in ss], out, sess.cap, n, step * 2, sess.res, g, sess.ws, sess.ws_bytes) == 0
    assert sess.result()["status"] == nz.ERR_MISMATCH
    assert nz.nz_reduce_k_step(ds, [s.size for s in ss], out, sess.cap, n, float("nan"), sess.res, g, sess.ws, sess.ws_bytes) == nz.ERR_INVALID


def test_captured_in_a_hip_graph(nz):
    """nz_reduce_k reads its host arrays of pointers and sizes during the call only, and only launches kernels: it can be
    recorded into a HIP graph.  Replays, with eager work in between, must reproduce the oracle's stream every time."""
    import torch
    n, eb, chunk, k = 200000, 1e-4, 65536, 5
    g, o = nz.make_opts(chunk_elems=chunk), oracle.make_opts(chunk_elems=chunk)
    ss = [oracle.compress(W.gradient_like(n, seed=480 + p), eb, o)[0] for p in range(k)]
    ref, ores, orc = oracle.reduce_k(ss, n, eb, o)
    assert orc == 0
    sess = nz.Session(n, g, "cuda:0", reduce=True)
    ds = [_dev(np.concatenate([s, np.zeros((-s.size) % 16, np.uint8)])) for s in ss]
    sizes = [s.size for s in ss]
    out = sess.new_stream_buffer()

    def work():
        assert nz.nz_reduce_k(ds, sizes, out, sess.cap, n, eb, sess.res, g, sess.ws, sess.ws_bytes) == 0

    work()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        work()
        graph.capture_end()
    for rep in range(3):
        out.zero_(); sess.res.zero_(); sess.ws.zero_()          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        r = sess.result()
        assert r["status"] == 0 and r["bytes"] == ores.bytes, rep
        assert np.array_equal(out[:r["bytes"]].cpu().numpy(), ref), rep


@pytest.mark.parametrize("predictor", [0, 1], ids=["plain", "delta"])
def test_garbage_in_an_operand(nz, predictor):
    """Byte flips anywhere behind the stream header of one operand (HUFFMAN, FIXEDLEN and RAW frames), the damaged
    operand in any position: never a fault, the oracle's verdict, and -- where the damage cannot be told from valid
    data -- the oracle's stream."""
    n = 5 * 16384 + 777
    eb = 1e-4
    kw = dict(chunk_elems=16384, predictor=predictor)
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    x = np.concatenate([W.gradient_like(2 * 16384, seed=191), W.sweep_payload("uniform", 2 * 16384, 192),
                        W.gradient_like(16384 + 777, seed=193)])
    x[3 * 16384 + 5] = np.inf                                           # frame 3 is RAW
    s = oracle.compress(x, eb, o)[0]
    others = [oracle.compress(W.gradient_like(n, seed=194 + p), eb, o)[0] for p in range(3)]
    rng = np.random.default_rng(23 + predictor)
    base = 64 + 8 * 6
    n_rejected = n_accepted = 0
    for trial in range(48):
        t = s.copy()
        for _ in range(int(rng.integers(1, 4))):
            t[int(rng.integers(base, s.size))] ^= int(rng.integers(1, 256))
        pos = trial % 4
        ops = list(others); ops.insert(pos, t)
        ref, ores, orc = oracle.reduce_k(ops, n, eb, o)
        rc, r, got = gpu_reduce_k(nz, ops, n, eb, g)
        assert rc == 0 and r["status"] == orc, (trial, pos, r, orc)
        if orc == 0:
            assert r["bytes"] == ores.bytes and np.array_equal(got, ref), (trial, pos)
            n_accepted += 1
        else:
            assert r["bytes"] == 0
            n_rejected += 1
    assert n_rejected >= 2 and n_accepted >= 2
