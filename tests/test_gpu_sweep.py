"""Seeded differential sweep: random sizes, frame geometries, alphabets, pinned codecs, gates, predictor and data kinds
through every entry point family (compress, decompress, two-stream / ring-step / k-ary reduce, sampled arbitration on
input and on the ring step, stochastic quantizer and its ring step), each result against the oracle to the bars of
the per-entry-point tests whose checkers are reused here."""
import numpy as np
import pytest

import oracle
import test_gpu_parity as P
import test_gpu_rea as R
import test_gpu_reduce_k as K
import test_gpu_sr as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nz(gpu_device):
    from paper_2605_12396_amd import binding
    binding.lib()
    return binding


def _data(rng, n, eb):
    kind = rng.choice(["lap", "lap", "lap", "uni", "zero", "const", "smooth", "mix"])
    scale = eb * float(rng.choice([0.3, 2, 10, 50, 300, 3000, 20000]))
    if kind == "lap":
        x = rng.laplace(0, scale, n)
    elif kind == "uni":
        x = rng.uniform(-scale * 3, scale * 3, n)
    elif kind == "zero":
        x = np.zeros(n)
    elif kind == "const":
        x = np.full(n, scale * 1.7)
    elif kind == "smooth":
        x = scale * 20 * np.sin(np.arange(n) / float(rng.uniform(5, 500))) + rng.normal(0, eb, n)
    else:
        x = rng.laplace(0, scale, n)
        m = rng.random(n) < 0.02
        x[m] = rng.laplace(0, scale * 100, int(m.sum()))
    x = x.astype(np.float32)
    r = rng.random()
    if r < 0.12:
        x[rng.integers(0, n)] = np.nan
    elif r < 0.2:
        x[rng.integers(0, n)] = np.inf
    elif r < 0.3:
        x[rng.integers(0, n)] = np.float32(eb * 1e6)
    return x


@pytest.mark.parametrize("seed", range(60))
def test_every_entry_point_on_random_cases(nz, seed):
    rng = np.random.default_rng(900000 + seed)
    n = int(rng.choice([1, 2, 5, 63, 255, 256, 257, 1000, 4097, 65535, 65536, 65537, 100001, 262144, 300007, 700001]))
    if rng.random() < 0.3:
        n = int(rng.integers(1, 3000))
    chunk = int(rng.choice([1, 3, 16, 255, 256, 257, 1000, 4096, 16384, 65536, 65537, 100003, 131072, 262144, 1 << 20]))
    if n // chunk > 5000:
        chunk = max(chunk, n // 2000)
    alphabet = int(rng.choice([2, 4, 16, 64, 256, 256, 256, 1024]))
    kw = dict(chunk_elems=chunk, alphabet=alphabet, force_codec=int(rng.choice([-1, -1, -1, -1, 0, 1, 2])),
              min_gain_permil=int(rng.choice([0, 0, 0, 300, 700, 999])), huff_min_bytes=int(rng.choice([0, 0, 0, 4096, 1 << 20])),
              predictor=int(rng.choice([0, 0, 1])))
    eb = float(rng.choice([1e-2, 1e-3, 1e-4, 1e-5]))
    src_kw = dict(chunk_elems=chunk, alphabet=alphabet, predictor=kw["predictor"])
    xs = [_data(rng, n, eb) for _ in range(4)]
    ref, _ = P.check_compress(nz, xs[0], eb, **kw)
    P.check_decompress(nz, ref, xs[0], eb, **kw)
    plain = [oracle.compress(x, eb, oracle.make_opts(**src_kw))[0] for x in xs]
    g, o = nz.make_opts(**kw), oracle.make_opts(**kw)
    r0, ores, orc = oracle.reduce_frames(plain[0], plain[1], n, eb, o)
    rc, r, got = P.gpu_reduce(nz, plain[0], plain[1], n, eb, g)
    assert rc == 0 and orc == 0 and r["status"] == 0 and r["bytes"] == ores.bytes and P._first_diff(got, r0) == -1
    P._check_reduce_local(nz, plain[0], xs[1], eb, **kw)
    K.check(nz, plain[:int(rng.integers(2, 5))], n, eb, **kw)
    if kw["predictor"]:
        return                          # (the sampled arbitration and the stochastic quantizer are built without it)
    ropts = None
    if rng.random() < 0.5:
        ropts = (int(rng.choice([256, 4096, 65536])), int(rng.choice([0, 0, 8192])), int(rng.choice([0, 0, 5, 200])),
                 int(rng.choice([0, 1000])), int(rng.choice([0, 3])), int(rng.choice([0, 2000])), int(rng.choice([0, 6])), 0)
    with_ctx = bool(rng.random() < 0.85)
    R.check_rea(nz, xs[0], eb, ropts=ropts, with_ctx=with_ctx, **kw)
    R.check_ring_rea(nz, xs[2], xs[0], eb, ropts=ropts, with_ctx=with_ctx, a_kw=dict(chunk_elems=chunk, alphabet=alphabet), **kw)
    fin = [x for x in xs if np.isfinite(x).all()]
    if not fin:
        return
    step = float(np.float32(max(oracle.qsgd_step(x, int(rng.choice([4, 200, 30000]))) for x in fin)))
    if step < 2.0 ** -100:
        return
    S.check_sr(nz, xs[0], step, seed, **kw)
    a1, _, rc1 = oracle.compress_sr(xs[1], step, seed + 1, oracle.make_opts(**src_kw))
    ref2, ores2, orc2 = oracle.reduce_local_sr(a1, xs[2], step, seed + 2, o)
    rc2, r2, got2 = S._gpu_reduce_local_sr(nz, a1, xs[2], step, seed + 2, g)
    assert rc1 == 0 and orc2 == 0 and rc2 == 0 and r2["status"] == 0 and r2["bytes"] == ores2.bytes
    assert np.array_equal(got2, ref2)
