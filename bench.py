#!/usr/bin/env python3
"""Benchmark of the per-rank compression path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input already resident in HBM:
nz_compress(message) -> nz_decompress(stream) -> nz_reduce_frames(stream, peer stream), on the headline
workload (64 Mi fp32 gradient-like values, eb = 1e-4 x range, 1 MiB frames).  `value` is the fp32 input bytes
the three stages handle per step (3 x 4n) divided by the step time.  Per-stage GB/s, the compression ratio,
the roofline record of the dominant kernel (HIP events recorded by the library between its kernels) and the
CPU oracle timed on this host's cores are reported in the same JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def make_workload(name):
    import numpy as np
    from paper_2605_12396_amd import workloads as W
    if name == "c2":
        n = 1 << 26
        x = W.gradient_like(n, seed=2)
        peer = W.gradient_like(n, seed=102)
        eb = W.abs_bound_from_rel(x, 1e-4)
        desc = "config2: 64Mi fp32 Laplace(0,1e-3)+1% Laplace(0,1e-1) outliers, eb=1e-4*range, 1MiB frames"
        chunk = 262144
    elif name == "c1":
        x = W.smooth_field((256, 64, 64), seed=1)
        peer = W.smooth_field((256, 64, 64), seed=11)
        n, eb, chunk = x.size, 1e-4, 16384
        desc = "config1: smooth 256x64x64 fp32 field, eb=1e-4, 64KiB frames"
    elif name == "c4":
        n = 1 << 25
        x = W.gradient_like(n, seed=40, outlier_frac=0.0)
        peer = W.gradient_like(n, seed=41, outlier_frac=0.0)
        eb, chunk = 1e-5, 262144
        desc = "config4 (one ring step): 32Mi fp32 Laplace(0,1e-3) per peer, eb=1e-5, 1MiB frames"
    else:
        raise SystemExit("unknown workload %r" % name)
    return dict(name=name, desc=desc, n=n, x=x, peer=peer, eb=float(np.float32(eb)), chunk=chunk)


def cpu_baseline(wl, alphabet=256):
    """The oracle as it stands, single thread, on the whole headline message (about 10-15 s of CPU work)."""
    import oracle
    n = wl["n"]
    o = oracle.make_opts(chunk_elems=wl["chunk"], alphabet=alphabet)
    t0 = time.perf_counter()
    s, res, rc = oracle.compress(wl["x"], wl["eb"], o)
    t1 = time.perf_counter()
    y, _, rc2 = oracle.decompress(s, n, wl["eb"])
    t2 = time.perf_counter()
    sp, _, _ = oracle.compress(wl["peer"], wl["eb"], o)
    t3 = time.perf_counter()
    r, _, rc3 = oracle.reduce_frames(s, sp, n, wl["eb"], o)
    t4 = time.perf_counter()
    assert rc == 0 and rc2 == 0 and rc3 == 0
    step = (t1 - t0) + (t2 - t1) + (t4 - t3)
    gb = 4.0 * n / 1e9
    par = cpu_baseline_frame_parallel(wl, o)
    return dict(value=3 * gb / step, unit="GB/s", cores=1, kind="oracle", frame_parallel=par,
                sample="whole %s message (%d elements): compress %.2fs, decompress %.2fs, reduce %.2fs" %
                       (wl["name"], n, t1 - t0, t2 - t1, t4 - t3),
                compress_GBps=gb / (t1 - t0), decompress_GBps=gb / (t2 - t1), reduce_GBps=gb / (t4 - t3)), s, r


def cpu_baseline_frame_parallel(wl, o):
    """The same oracle on all host cores of the GPU's share: frames are independent, so the message is cut into runs of
    whole frames and every thread runs the unchanged single-threaded oracle on its run (a stream per run; the calls
    release the interpreter lock).  Reported beside the single-thread figure, never instead of it."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    n, chunk, eb = wl["n"], wl["chunk"], wl["eb"]
    frames = (n + chunk - 1) // chunk
    threads = max(1, min(16, os.cpu_count() or 1, frames))
    cuts = [min(n, chunk * ((frames * t) // threads)) for t in range(threads + 1)]
    runs = [(cuts[t], cuts[t + 1]) for t in range(threads) if cuts[t + 1] > cuts[t]]
    x, peer = wl["x"], wl["peer"]
    with ThreadPoolExecutor(len(runs)) as pool:
        t0 = time.perf_counter()
        ss = list(pool.map(lambda r: oracle.compress(x[r[0]:r[1]], eb, o)[0], runs))
        t1 = time.perf_counter()
        list(pool.map(lambda a: oracle.decompress(a[0], a[1][1] - a[1][0], eb)[0], zip(ss, runs)))
        t2 = time.perf_counter()
        sp = list(pool.map(lambda r: oracle.compress(peer[r[0]:r[1]], eb, o)[0], runs))
        t3 = time.perf_counter()
        list(pool.map(lambda a: oracle.reduce_frames(a[0], a[1], a[2][1] - a[2][0], eb, o)[0], zip(ss, sp, runs)))
        t4 = time.perf_counter()
    gb = 4.0 * n / 1e9
    return dict(value=3 * gb / ((t1 - t0) + (t2 - t1) + (t4 - t3)), unit="GB/s", cores=len(runs),
                compress_GBps=gb / (t1 - t0), decompress_GBps=gb / (t2 - t1), reduce_GBps=gb / (t4 - t3))


def oracle_decompress(stream, n, eb):
    import oracle
    y, _, rc = oracle.decompress(stream, n, eb)
    assert rc == 0
    return y


def read_traffic(path, workload, kernel):
    """HBM bytes per launch of `kernel` (fetch + write, calibrated against a copy kernel) from the committed
    counter summary: lines of the form `<workload> <stage>/<kernel> fetch_bytes write_bytes`.  None if absent."""
    try:
        with open(path) as f:
            for line in f:
                t = line.split()
                if len(t) >= 4 and not line.startswith("#") and t[0] == workload and t[1] == kernel:
                    return float(t[2]) + float(t[3])
    except OSError:
        pass
    return None


def run_c5_overlap(args):
    """Config 5: a message compressed slice by slice on one HIP stream while the finished slices are copied to
    pinned host memory on a second stream (the copy stands in for the transport).  Prints one JSON line per
    payload kind with the serialized time, the overlapped time, the copy-only time and the exposed compression
    time = overlapped - copy-only.  Not part of the headline metric."""
    import numpy as np
    import torch
    from paper_2605_12396_amd import binding as nz, workloads as W

    dev = torch.device("cuda:0")
    eb = 1e-4
    s_comp, s_copy = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)     # default priority
    kinds = ("uniform", "laplace", "sinusoid")
    # message sizes 64 KB .. 1 GB in powers of 4, the payload kind rotating with the size; 64 KiB frames up to 4 MB,
    # 1 MiB frames above; slices of 16 MB (smaller messages are one slice)
    for k, (n, kind) in enumerate([(16384 << (2 * i), kinds[i % 3]) for i in range(8)] +
                                  [(1 << 26, "laplace"), (1 << 26, "uniform"), (1 << 26, "sinusoid")]):
        if 4 * n > args.c5_max_bytes:
            continue
        chunk = 16384 if 4 * n <= (4 << 20) else 262144
        slice_n = min(n, 1 << 22)
        n_slices = n // slice_n
        opts = nz.make_opts(chunk_elems=chunk, alphabet=args.alphabet)
        x = torch.from_numpy(W.sweep_payload(kind, n, 50 + k)).to(dev)
        cap = nz.nz_compress_bound(slice_n, opts)
        wsb = nz.nz_workspace_bytes(slice_n, opts)
        outs = [torch.empty(cap, dtype=torch.uint8, device=dev) for _ in range(2)]       # two banks
        wss = [torch.empty(wsb, dtype=torch.uint8, device=dev) for _ in range(2)]
        ress = [torch.zeros(nz.RESULT_BYTES, dtype=torch.uint8, device=dev) for _ in range(n_slices)]
        host = torch.empty(cap, dtype=torch.uint8, pin_memory=True)
        host_res = [torch.empty(nz.RESULT_BYTES, dtype=torch.uint8, pin_memory=True) for _ in range(n_slices)]
        sizes = []

        def compress_slice(i, stream):
            nz.nz_compress(x[i * slice_n:(i + 1) * slice_n], slice_n, eb, outs[i % 2], cap, ress[i], opts, wss[i % 2], wsb,
                           stream=stream)

        # sizes once (untimed), so that the copy-only leg moves exactly the same bytes
        for i in range(n_slices):
            compress_slice(i, torch.cuda.current_stream())
            sizes.append(nz.read_result(ress[i])["bytes"])
        torch.cuda.synchronize()

        def serialized():
            t0 = time.perf_counter()
            for i in range(n_slices):
                compress_slice(i, s_comp)
                s_comp.synchronize()
                with torch.cuda.stream(s_copy):
                    host[:sizes[i]].copy_(outs[i % 2][:sizes[i]], non_blocking=True)
                s_copy.synchronize()
            return time.perf_counter() - t0

        def copy_only():
            t0 = time.perf_counter()
            with torch.cuda.stream(s_copy):
                for i in range(n_slices):
                    host[:sizes[i]].copy_(outs[i % 2][:sizes[i]], non_blocking=True)
            s_copy.synchronize()
            return time.perf_counter() - t0

        def overlapped():
            # slice i is compressed into bank i%2 while slice i-1 leaves bank (i-1)%2; a bank is reused only after
            # its copy has finished; the host learns each slice's byte count from a 32-byte copy of the result record
            ev_done = [torch.cuda.Event() for _ in range(n_slices)]
            ev_copied = [torch.cuda.Event() for _ in range(n_slices)]
            t0 = time.perf_counter()
            for i in range(n_slices):
                if i >= 2:
                    s_comp.wait_event(ev_copied[i - 2])
                compress_slice(i, s_comp)
                with torch.cuda.stream(s_comp):
                    host_res[i].copy_(ress[i], non_blocking=True)
                    ev_done[i].record(s_comp)
                if i >= 1:
                    j = i - 1
                    ev_done[j].synchronize()
                    nb = int(host_res[j].numpy()[:8].view(np.uint64)[0])
                    with torch.cuda.stream(s_copy):
                        host[:nb].copy_(outs[j % 2][:nb], non_blocking=True)
                        ev_copied[j].record(s_copy)
            j = n_slices - 1
            ev_done[j].synchronize()
            nb = int(host_res[j].numpy()[:8].view(np.uint64)[0])
            with torch.cuda.stream(s_copy):
                host[:nb].copy_(outs[j % 2][:nb], non_blocking=True)
            s_copy.synchronize(); s_comp.synchronize()
            return time.perf_counter() - t0

        for f in (serialized, copy_only, overlapped):
            f()                                                   # warm-up
        reps = max(3, min(args.steps, 10)) if n >= (1 << 24) else 20
        t_ser = min(serialized() for _ in range(reps))
        t_cpy = min(copy_only() for _ in range(reps))
        t_ovl = min(overlapped() for _ in range(reps))
        total = float(sum(sizes))
        print(json.dumps(dict(metric="exposed compression time, sliced compress overlapped with D2H copy (config 5)",
                              config=dict(workload="c5 %s, %d-byte message, %d slice(s) of %d bytes, eb=1e-4, %d-element frames" %
                                                   (kind, 4 * n, n_slices, 4 * slice_n, chunk), alphabet=args.alphabet),
                              data="synthetic", n_gpus=1, compressed_bytes=total, compression_ratio=4.0 * n / total,
                              serialized_ms=t_ser * 1e3, copy_only_ms=t_cpy * 1e3, overlapped_ms=t_ovl * 1e3,
                              exposed_compression_ms=(t_ovl - t_cpy) * 1e3,
                              serialized_over_overlapped=t_ser / t_ovl)))


def run_c3_bounds(args):
    """Config 3: Gaussian random field 512^3 (P(k) ~ k^-3, unit variance), value-range-relative bound swept over
    1e-2, 1e-3, 1e-4, 1 MiB frames: compression ratio against compress / decompress throughput per bound.  The field
    is drawn on the GPU (torch, seeded) with the recipe of workloads.gaussian_random_field; a 4-frame sample is
    compared with the oracle.  One JSON line per bound; not part of the headline metric."""
    import numpy as np
    import torch
    import oracle
    from paper_2605_12396_amd import binding as nz

    dev = torch.device("cuda:0")
    N = args.c3_side
    gen = torch.Generator(device=dev); gen.manual_seed(3)
    f = torch.randn((N, N, N), generator=gen, device=dev, dtype=torch.float32)
    F = torch.fft.rfftn(f)
    k1 = torch.fft.fftfreq(N, device=dev) * N
    kz = torch.fft.rfftfreq(N, device=dev) * N
    k = torch.sqrt(k1[:, None, None] ** 2 + k1[None, :, None] ** 2 + kz[None, None, :] ** 2)
    k[0, 0, 0] = 1.0
    amp = k ** -1.5
    amp[0, 0, 0] = 0.0
    F *= amp
    del k, amp
    f = torch.fft.irfftn(F, s=(N, N, N))
    del F
    f = ((f - f.mean()) / f.std()).float().contiguous().view(-1)
    n = f.numel()
    rng = float(f.max() - f.min())
    opts = nz.make_opts(chunk_elems=262144, alphabet=args.alphabet)
    sess = nz.Session(n, opts, dev)
    out = sess.new_stream_buffer()
    y = torch.empty_like(f)
    gb = 4.0 * n / 1e9
    for rel in (1e-2, 1e-3, 1e-4):
        eb = float(np.float32(rel * rng))
        def timed(fn, reps):
            fn(); torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record(); torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        reps = max(3, min(args.steps, 10))
        t_c = timed(lambda: sess.compress(f, eb, out=out), reps)
        r = sess.result()
        assert r["status"] == 0
        nbytes = r["bytes"]
        t_d = timed(lambda: sess.decompress(out, nbytes, n, eb, out=y), reps)
        assert sess.result()["status"] == 0
        err = float((y.double() - f.double()).abs().max())
        # first four frames against the oracle: same bytes
        xs = f[:4 * 262144].cpu().numpy()
        ref, ores, orc = oracle.compress(xs, eb, oracle.make_opts(chunk_elems=262144, alphabet=args.alphabet))
        s4 = nz.Session(xs.size, opts, dev)
        rc, o4 = s4.compress(f[:4 * 262144], eb)
        r4 = s4.result()
        same = bool(orc == 0 and r4["bytes"] == ores.bytes and (o4[:r4["bytes"]].cpu().numpy() == ref).all())
        print(json.dumps(dict(metric="compression ratio vs throughput per bound (config 3)", n_gpus=1, data="synthetic",
                              config=dict(workload="c3: Gaussian random field %d^3, P(k)~k^-3, REL=%g x range, 1MiB frames" % (N, rel),
                                          alphabet=args.alphabet, eb=eb),
                              compression_ratio=4.0 * n / nbytes, compress_GBps=gb / (t_c * 1e-3), decompress_GBps=gb / (t_d * 1e-3),
                              compress_ms=t_c, decompress_ms=t_d, max_abs_err=err, bound_holds=bool(err <= eb),
                              frames=dict(raw=r["n_raw"], fixed=r["n_fixed"], huffman=r["n_huff"]),
                              first_4_frames_match_oracle=same)))


def run_predictor(args):
    """The delta predictor on the codes (opts.predictor = 1) against the plain path: compression ratio and compress /
    decompress throughput on three inputs -- the config-1 field (3-D, its fastest axis has only 64 points per line, so
    a 1-D difference removes little), a 256^3 cut of the config-3 recipe at REL 1e-3, and a smooth 1-D signal
    (sin(i/300) + N(0, 1e-4), the case a 1-D predictor is made for).  The first frames of every run are compared with
    the oracle.  One JSON line per (input, predictor); not part of the headline metric."""
    import numpy as np
    import torch
    import oracle
    from paper_2605_12396_amd import binding as nz, workloads as W

    dev = torch.device("cuda:0")
    rng = np.random.default_rng(7)
    n1d = 1 << 24
    inputs = [("c1: 256x64x64 smooth field + N(0,1e-3), eb=1e-4, 64KiB frames", W.smooth_field((256, 64, 64), seed=1), 1e-4, 16384),
              ("c3 recipe at 256^3, REL=1e-3 x range, 1MiB frames", W.gaussian_random_field(256, seed=3).reshape(-1), None, 262144),
              ("smooth 1-D: sin(i/300) + N(0,1e-4), 16Mi elements, eb=1e-4, 1MiB frames",
               (np.sin(np.arange(n1d) / 300.0) + 1e-4 * rng.normal(size=n1d)).astype(np.float32), 1e-4, 262144)]
    for desc, x, eb, chunk in inputs:
        x = np.ascontiguousarray(x, dtype=np.float32)
        n = x.size
        eb = float(np.float32(eb if eb is not None else 1e-3 * float(x.max() - x.min())))
        f = torch.from_numpy(x).to(dev)
        y = torch.empty_like(f)
        gb = 4.0 * n / 1e9
        for pred in (0, 1):
            opts = nz.make_opts(chunk_elems=chunk, alphabet=args.alphabet, predictor=pred)
            sess = nz.Session(n, opts, dev)
            out = sess.new_stream_buffer()

            def timed(fn, reps):
                fn(); torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    fn()
                e1.record(); torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps
            reps = max(3, min(args.steps, 20))
            t_c = timed(lambda: sess.compress(f, eb, out=out), reps)
            r = sess.result()
            assert r["status"] == 0
            nbytes = r["bytes"]
            t_d = timed(lambda: sess.decompress(out, nbytes, n, eb, out=y), reps)
            assert sess.result()["status"] == 0
            err = float((y.double() - f.double()).abs().max())
            m = min(n, 4 * chunk)
            ref, ores, orc = oracle.compress(x[:m], eb, oracle.make_opts(chunk_elems=chunk, alphabet=args.alphabet, predictor=pred))
            s4 = nz.Session(m, opts, dev)
            rc, o4 = s4.compress(f[:m], eb)
            r4 = s4.result()
            same = bool(orc == 0 and r4["bytes"] == ores.bytes and (o4[:r4["bytes"]].cpu().numpy() == ref).all())
            print(json.dumps(dict(metric="compression ratio and throughput with / without the delta predictor", n_gpus=1,
                                  data="synthetic", config=dict(workload=desc, predictor=pred, alphabet=args.alphabet, eb=eb),
                                  compression_ratio=4.0 * n / nbytes, compress_GBps=gb / (t_c * 1e-3),
                                  decompress_GBps=gb / (t_d * 1e-3), compress_ms=t_c, decompress_ms=t_d, max_abs_err=err,
                                  bound_holds=bool(err <= eb), frames=dict(raw=r["n_raw"], fixed=r["n_fixed"], huffman=r["n_huff"]),
                                  first_frames_match_oracle=same)))


def run_c4_ring(args):
    """Config 4: one rank's share of a reduce-scatter ring over 8 peers: 7 fused steps acc = reduce(acc, peer_p) on
    32 Mi-element messages (eb = 1e-5, 1 MiB frames), peers pre-compressed untimed.  Also the ring-step variant in
    which the rank adds its own fp32 data (nz_reduce_local).  Prints one JSON line; not part of the headline metric."""
    import numpy as np
    import torch
    from paper_2605_12396_amd import binding as nz, workloads as W

    dev = torch.device("cuda:0")
    n, eb, peers = 1 << 25, 1e-5, 8
    opts = nz.make_opts(chunk_elems=262144, alphabet=args.alphabet)
    sess = nz.Session(n, opts, dev, reduce=True)
    msgs = [torch.from_numpy(W.gradient_like(n, seed=40 + p, outlier_frac=0.0)).to(dev) for p in range(peers)]
    streams, sizes = [], []
    for m in msgs:
        rc, out = sess.compress(m, eb)
        r = sess.result()
        assert rc == 0 and r["status"] == 0
        streams.append(out); sizes.append(r["bytes"])
    bufs = [sess.new_stream_buffer() for _ in range(2)]

    def chain(local):
        acc, acc_bytes, per_step = streams[0], sizes[0], []
        for p in range(1, peers):
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            if local:
                rc, out = sess.reduce_local(acc, acc_bytes, msgs[p], n, eb, out=bufs[p % 2])
            else:
                rc, out = sess.reduce(acc, acc_bytes, streams[p], sizes[p], n, eb, out=bufs[p % 2])
            ev1.record()
            r = sess.result()                                     # synchronises: the next step needs the byte count
            assert rc == 0 and r["status"] == 0
            per_step.append(ev0.elapsed_time(ev1))
            acc, acc_bytes = out, r["bytes"]
        return per_step, acc_bytes

    chain(False); chain(True)                                     # warm-up
    reps = max(2, min(args.steps, 5))
    best = {}
    for local in (False, True):
        runs = [chain(local) for _ in range(reps)]
        steps_ms = [min(r[0][i] for r in runs) for i in range(peers - 1)]
        best[local] = (steps_ms, runs[0][1])
    # all eight contributions at once: every operand decoded once, the sum encoded once (nz_reduce_k); the result is
    # the chain's final stream byte for byte
    kout = sess.new_stream_buffer()
    def kary():
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        rc, _ = sess.reduce_k(streams, sizes, n, eb, out=kout)
        ev1.record()
        r = sess.result()
        assert rc == 0 and r["status"] == 0
        return ev0.elapsed_time(ev1), r["bytes"]
    kary()
    k_ms, k_bytes = min(kary() for _ in range(reps))
    with nz.KernelTrace(16) as tr:
        sess.reduce_k(streams, sizes, n, eb, out=kout)
        k_kernels = tr.kernel_ms()
    chain_ms, chain_bytes = chain(False)
    final = bufs[(peers - 1) % 2]
    k_equal = bool(k_bytes == chain_bytes and torch.equal(kout[:k_bytes], final[:chain_bytes]))
    gb = 4.0 * n / 1e9
    print(json.dumps(dict(metric="fused reduce ring step, GB/s of fp32 input per step (config 4)", unit="GB/s", n_gpus=1,
                          data="synthetic",
                          config=dict(workload="c4: 8 peers x 32Mi fp32 Laplace(0,1e-3), eb=1e-5, 1MiB frames, 7 steps",
                                      alphabet=args.alphabet),
                          input_compression_ratio=4.0 * n / sizes[0], final_compression_ratio=4.0 * n / best[False][1],
                          reduce_frames=dict(per_step_ms=best[False][0], total_ms=sum(best[False][0]),
                                             GBps=gb * (peers - 1) / (sum(best[False][0]) * 1e-3)),
                          reduce_local=dict(per_step_ms=best[True][0], total_ms=sum(best[True][0]),
                                            GBps=gb * (peers - 1) / (sum(best[True][0]) * 1e-3)),
                          reduce_k=dict(total_ms=k_ms, GBps=gb * peers / (k_ms * 1e-3),
                                        kernel_ms=dict(zip(["init", "stage_0"] + ["acc_%d" % p for p in range(1, peers - 1)] +
                                                           ["add_last", "fix", "codebook", "encode"], k_kernels)),
                                        stream_equals_chain=k_equal),
                          final_bytes_equal=bool(best[False][1] == best[True][1]))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2", help="c2 (headline) | c1 | c4 | c3 | c4ring | c5 | pred")
    ap.add_argument("--alphabet", type=int, default=256, help="Huffman alphabet K (power of two, 2..1024)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true", help="also time the step replayed from a HIP graph (reported beside ms_per_step)")
    ap.add_argument("--rotate", type=int, default=3, help="number of distinct input / stream copies cycled through")
    ap.add_argument("--only", default="", help="profiling aid: time only this stage (compress|decompress|reduce|compress_rea)")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="profiling aid: also run this many plain 4n-byte copy kernels (counter calibration)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "hbm_traffic_c2.txt"),
                    help="text summary of the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see pmc_summary.py)")
    ap.add_argument("--c3-side", type=int, default=512, help="c3: side of the cubic random field")
    ap.add_argument("--c5-max-bytes", type=int, default=1 << 30, help="c5: largest message of the size sweep")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures the one-GPU hot path only: run with --gpus 1 "
                         "(no collectives or second GPU are part of this build)")

    if args.workload == "c5":
        return run_c5_overlap(args)
    if args.workload == "c4ring":
        return run_c4_ring(args)
    if args.workload == "c3":
        return run_c3_bounds(args)
    if args.workload == "pred":
        return run_predictor(args)

    import numpy as np
    import torch
    from paper_2605_12396_amd import binding as nz

    nz.lib()
    dev = torch.device("cuda:0")
    wl = make_workload(args.workload)
    n, eb = wl["n"], wl["eb"]
    opts = nz.make_opts(chunk_elems=wl["chunk"], alphabet=args.alphabet)
    sess = nz.Session(n, opts, dev, reduce=True)

    # R copies of everything a stage reads, so that no stage finds its input in the caches: step i compresses copy
    # i % R of the message and decompresses / reduces the streams in buffers (i + 1) % R, which were written R - 1
    # steps (several times the 256 MB Infinity Cache) earlier.  All copies hold the same bytes.
    R = max(1, args.rotate)
    xs = [torch.from_numpy(wl["x"]).to(dev) for _ in range(R)]
    xpeer = torch.from_numpy(wl["peer"]).to(dev)
    outs = [sess.new_stream_buffer() for _ in range(R)]
    peers = [sess.new_stream_buffer() for _ in range(R)]
    red_out = sess.new_stream_buffer()
    y = torch.empty(n, dtype=torch.float32, device=dev)

    for k in range(R):
        rc, _ = sess.compress(xpeer, eb, out=peers[k])
        r = sess.result()
        assert rc == 0 and r["status"] == 0
        peer_bytes = r["bytes"]
        rc, _ = sess.compress(xs[k], eb, out=outs[k])
        r0 = sess.result()
        assert rc == 0 and r0["status"] == 0
        stream_bytes = r0["bytes"]

    # the sampled-arbitration compress (Algorithm 1 taken literally; not part of `value`): context from the first
    # 64 KiB-sample's worth of the message, one pass over the input, frames in RAW-sized slots
    ctx = torch.zeros(nz.nz_context_bytes(), dtype=torch.uint8, device=dev)
    assert nz.nz_context_build(xs[0], min(n, 65536), eb, opts, ctx, sess.ws, sess.ws_bytes) == 0
    rea_out = torch.empty(sess.cap, dtype=torch.uint8, device=dev)
    rea_res = torch.zeros(48, dtype=torch.uint8, device=dev)
    rea_wsb = nz.nz_rea_workspace_bytes(n, opts)
    rea_ws = torch.empty(rea_wsb, dtype=torch.uint8, device=dev)

    def compress_rea_call(k):
        return nz.nz_compress_rea(xs[k], n, eb, ctx, rea_out, sess.cap, rea_res, opts, None, rea_ws, rea_wsb)

    # the ring step with the sampled arbitration on the way out (not part of `value` either)
    rr_wsb = nz.nz_reduce_rea_workspace_bytes(n, opts)
    rr_ws = torch.empty(rr_wsb, dtype=torch.uint8, device=dev)
    rr_res = torch.zeros(48, dtype=torch.uint8, device=dev)
    rr_out = torch.empty(sess.cap, dtype=torch.uint8, device=dev)

    def reduce_local_rea_call(k2):
        return nz.nz_reduce_local_rea(outs[k2], stream_bytes, xpeer, n, eb, ctx, rr_out, sess.cap, rr_res, opts, None, rr_ws, rr_wsb)

    def step(i):
        k, k2 = i % R, (i + 1) % R
        a = b = c = 0
        if args.only == "compress_rea":
            return compress_rea_call(k)
        if args.only in ("", "decompress"):
            b = sess.decompress(outs[k2], stream_bytes, n, eb, out=y)[0]
        if args.only in ("", "reduce"):
            c = sess.reduce(outs[k2], stream_bytes, peers[k2], peer_bytes, n, eb, out=red_out)[0]
        if args.only in ("", "compress"):
            a = sess.compress(xs[k], eb, out=outs[k])[0]
        return a | b | c

    for _ in range(args.calib_copy):          # elementwise kernel reading 4n bytes and writing 4n bytes
        torch.add(xs[0], 0.0, out=y)
    for i in range(args.warmup):
        assert step(i) == 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    # the same step replayed from a HIP graph (launch-bound small messages): one capture of step 0, `steps` replays
    graph_ms = None
    if args.graph and not args.only:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.capture_begin()
            step(0)
            graph.capture_end()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        tg0 = time.perf_counter()
        for i in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg0) * 1e3 / args.steps
    if args.only:
        print(json.dumps(dict(only=args.only, ms_per_step=ms_per_step, GBps=4.0 * n / 1e9 / (ms_per_step * 1e-3))))
        return
    sess.reduce(outs[0], stream_bytes, peers[0], peer_bytes, n, eb, out=red_out)
    rr = sess.result()
    assert rr["status"] == 0
    reduce_bytes = rr["bytes"]

    # per-stage and per-kernel times from HIP events the library records on its own stream between its kernels
    names = {"compress": ["stats", "codebook", "encode"], "decompress": ["decode", "finish"],
             "reduce": ["init", "stage_a", "add_b", "fix", "codebook", "encode"],
             "reduce_local": ["init", "add_local", "fix", "codebook", "encode"],
             "compress_rea": ["encode", "finish"],
             "reduce_local_rea": ["init", "add_local", "fix", "encode", "finish"]}
    acc = {k: [0.0] * len(v) for k, v in names.items()}
    reps = max(5, min(args.steps, 20))

    def compress_rea(k):
        return compress_rea_call(k)
    assert compress_rea(0) == 0
    rea = nz.read_rea_result(rea_res)
    assert rea["status"] == 0
    with nz.KernelTrace(8) as tr:
        for i in range(reps):
            k, k2 = i % R, (i + 1) % R
            sess.decompress(outs[k2], stream_bytes, n, eb, out=y)
            for j, t in enumerate(tr.kernel_ms()):
                acc["decompress"][j] += t
            sess.reduce(outs[k2], stream_bytes, peers[k2], peer_bytes, n, eb, out=red_out)
            for j, t in enumerate(tr.kernel_ms()):
                acc["reduce"][j] += t
            # ring-step variant (not part of `value`): incoming stream + the rank's own fp32 data
            sess.reduce_local(outs[k2], stream_bytes, xpeer, n, eb, out=red_out)
            for j, t in enumerate(tr.kernel_ms()):
                acc["reduce_local"][j] += t
            sess.compress(xs[k], eb, out=outs[k])
            for j, t in enumerate(tr.kernel_ms()):
                acc["compress"][j] += t
            compress_rea(k2)
            for j, t in enumerate(tr.kernel_ms()):
                acc["compress_rea"][j] += t
            assert reduce_local_rea_call(k2) == 0
            for j, t in enumerate(tr.kernel_ms()):
                acc["reduce_local_rea"][j] += t
    kern = {st: {nm: acc[st][j] / reps for j, nm in enumerate(names[st])} for st in names}
    # frames on which the sampled plan committed another codec than the exact selector (mis-selection count)
    nfr = r0["n_frames"]
    offs_e = outs[0][64:64 + 8 * nfr].cpu().numpy().view(np.uint64).astype(np.int64)
    offs_r = rea_out[64:64 + 8 * nfr].cpu().numpy().view(np.uint64).astype(np.int64)
    cod_e = outs[0].cpu().numpy()[(offs_e + 4)]
    cod_r = rea_out.cpu().numpy()[(offs_r + 4)]
    misselected = (cod_e != cod_r).sum()
    # what a plain streaming kernel reaches on this machine: elementwise copy of 4 messages' worth of data per launch
    # (16n bytes read + 16n written), large enough that the launch gap does not matter
    copy_gbps = None
    if not args.calib_copy:                   # (a counter-calibration run keeps its copy kernels of one size only)
        big_in = torch.empty(4 * n, dtype=torch.float32, device=dev).normal_()
        big_out = torch.empty_like(big_in)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.add(big_in, 0.0, out=big_out)
        ev0.record()
        for i in range(5):
            torch.add(big_in, 0.0, out=big_out)
        ev1.record()
        torch.cuda.synchronize()
        del big_in, big_out
        copy_gbps = 2 * 16.0 * n / 1e9 / (ev0.elapsed_time(ev1) * 1e-3 / 5)
    stage_ms = {st: sum(kern[st].values()) for st in names}
    gb = 4.0 * n / 1e9
    cr = 4.0 * n / stream_bytes
    # Algorithmic bytes: what the method itself must move (fp32 in or out, compressed streams in or out), nothing
    # this implementation stages in between.  Per operation: compress 4n + S, decompress S + 4n, reduce
    # S_a + S_b + S_out, ring step S_in + 4n + S_out; per kernel: the part of those bytes that kernel touches.
    alg_op = {"compress": 4.0 * n + stream_bytes, "decompress": stream_bytes + 4.0 * n,
              "reduce": stream_bytes + peer_bytes + reduce_bytes, "reduce_local": stream_bytes + 4.0 * n + reduce_bytes,
              "compress_rea": 4.0 * n + rea["wire_bytes"]}
    rrea = nz.read_rea_result(rr_res)
    assert rrea["status"] == 0
    alg_op["reduce_local_rea"] = stream_bytes + 4.0 * n + rrea["wire_bytes"]
    alg = {("compress", "stats"): 4.0 * n, ("compress", "encode"): 4.0 * n + stream_bytes,
           ("decompress", "decode"): 4.0 * n + stream_bytes,
           ("reduce", "stage_a"): float(stream_bytes), ("reduce", "add_b"): float(peer_bytes),
           ("reduce", "encode"): float(reduce_bytes)}      # kernels of the step only (the ring-step variant is extra)
    dom = max(alg, key=lambda k: kern[k[0]][k[1]])
    dom_ms = kern[dom[0]][dom[1]]
    achieved = alg[dom] / (dom_ms * 1e-3) / 1e9
    roofline = dict(bound="hbm", kernel="%s/%s" % dom, achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=achieved / HBM_PEAK_GBPS, traffic=read_traffic(args.traffic_file, wl["name"], "%s/%s" % dom),
                    kernel_ms=dom_ms, algorithmic_bytes=alg[dom])
    # the three numbers per operation: fp32-input GB/s, algorithmic bytes / time as a fraction of the HBM peak, and
    # counter-measured HBM bytes (sum over the operation's kernels in the committed summary) / time
    ops = {}
    for st in names:
        t = stage_ms[st] * 1e-3
        traffic = None
        # every kernel of the operation that the counter summary lists (the tiny init kernel may be absent from it)
        parts = {nm: read_traffic(args.traffic_file, wl["name"], "%s/%s" % (st, nm)) for nm in names[st]}
        if all(v is not None for nm, v in parts.items() if nm != "init"):
            traffic = sum(v for v in parts.values() if v is not None)
        ops[st] = dict(ms=stage_ms[st], input_GBps=gb / t, input_frac_hbm=gb / t / HBM_PEAK_GBPS,
                       algorithmic_bytes=alg_op[st], algorithmic_GBps=alg_op[st] / 1e9 / t,
                       algorithmic_frac_hbm=alg_op[st] / 1e9 / t / HBM_PEAK_GBPS,
                       traffic_bytes=traffic, traffic_GBps=(traffic / 1e9 / t if traffic else None),
                       traffic_over_algorithmic=(traffic / alg_op[st] if traffic else None))

    out = dict(metric="compress / decompress / fused-reduce GB/s (fp32 input): bytes of the three stages over the step time", value=3 * gb / (ms_per_step * 1e-3),
               unit="GB/s", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms_per_step, graph_ms_per_step=graph_ms,
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="f32+i32", data="synthetic",
               config=dict(workload=wl["desc"], n_elems=n, chunk_elems=wl["chunk"], alphabet=args.alphabet, eb=eb,
                           rotate=R),
               stages=dict(compress_GBps=ops["compress"]["input_GBps"], decompress_GBps=ops["decompress"]["input_GBps"],
                           reduce_GBps=ops["reduce"]["input_GBps"],
                           compress_frac_hbm=ops["compress"]["input_frac_hbm"],
                           decompress_frac_hbm=ops["decompress"]["input_frac_hbm"],
                           reduce_frac_hbm=ops["reduce"]["input_frac_hbm"],
                           reduce_local_GBps=ops["reduce_local"]["input_GBps"],
                           copy_kernel_GBps=copy_gbps,
                           compression_ratio=cr, stream_bytes=stream_bytes, reduce_stream_bytes=reduce_bytes,
                           frames=dict(raw=r0["n_raw"], fixed=r0["n_fixed"], huffman=r0["n_huff"]),
                           kernel_ms=kern, operations=ops,
                           compress_rea=dict(GBps=ops["compress_rea"]["input_GBps"], frac_hbm=ops["compress_rea"]["input_frac_hbm"],
                                             wire_bytes=rea["wire_bytes"], compression_ratio=4.0 * n / rea["wire_bytes"],
                                             ratio_loss_vs_exact=1.0 - stream_bytes / rea["wire_bytes"],
                                             frames=dict(raw=rea["n_raw"], fixed=rea["n_fixed"], huffman=rea["n_huff"],
                                                         fallback=rea["n_fallback"]),
                                             frames_with_other_codec_than_exact=int(misselected)),
                           reduce_local_rea=dict(GBps=ops["reduce_local_rea"]["input_GBps"], frac_hbm=ops["reduce_local_rea"]["input_frac_hbm"],
                                                 wire_bytes=rrea["wire_bytes"], exact_bytes=reduce_bytes,
                                                 frames=dict(raw=rrea["n_raw"], fixed=rrea["n_fixed"], huffman=rrea["n_huff"],
                                                             fallback=rrea["n_fallback"]))),
               roofline=roofline)
    if not args.no_cpu_baseline:
        base, ref_stream, ref_reduced = cpu_baseline(wl, args.alphabet)
        out["cpu_baseline"] = base
        got = outs[0][:stream_bytes].cpu().numpy()
        out["bytes_match_oracle"] = bool(got.size == ref_stream.size and (got == ref_stream).all())
        sess.reduce(outs[0], stream_bytes, peers[0], peer_bytes, n, eb, out=red_out)
        got = red_out[:sess.result()["bytes"]].cpu().numpy()
        out["reduce_bytes_match_oracle"] = bool(got.size == ref_reduced.size and (got == ref_reduced).all())
        sess.decompress(outs[0], stream_bytes, n, eb, out=y)
        ref_y = oracle_decompress(ref_stream, n, eb)
        out["decompress_values_match_oracle"] = bool((y.cpu().numpy().view(np.uint32) == ref_y.view(np.uint32)).all())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
