"""The entry point that allocates nothing (nz_compress_static: the workspace is an array resident in the library)
against nz_compress with a caller-owned workspace, through the C ABI: same bytes and result record, on two calls in
a row of which the second is smaller (the array keeps the first call's contents)."""
import numpy as np
import pytest

from paper_2605_12396_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_nz_compress(gpu_device):
    import torch
    from paper_2605_12396_amd import binding as nz
    nz.lib()
    assert nz.nz_static_scratch_bytes() == 8 << 20
    eb = 1e-4
    for n, chunk, seed in ((3 * 262144 + 70001, 262144, 31), (100003, 16384, 32), (37, 16, 33)):
        g = nz.make_opts(chunk_elems=chunk)
        x = torch.from_numpy(W.gradient_like(n, seed=seed)).to(gpu_device)
        sess = nz.Session(n, g, gpu_device)
        rc, ref = sess.compress(x, eb)
        r_ref = sess.result()
        assert rc == 0 and r_ref["status"] == 0
        out = torch.zeros(sess.cap, dtype=torch.uint8, device=gpu_device)
        res = torch.zeros(nz.RESULT_BYTES, dtype=torch.uint8, device=gpu_device)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(gpu_device)
        rc = nz.nz_compress_static(x, n, eb, out, sess.cap, res, g)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(gpu_device) == before
        r = nz.read_result(res)
        assert rc == 0 and r == r_ref, (r, r_ref)
        assert torch.equal(out[:r["bytes"]], ref[:r["bytes"]])
    # a capacity error is reported the same way, and a message too large for the resident array is refused up front
    small = torch.zeros(4096, dtype=torch.uint8, device=gpu_device)
    rc = nz.nz_compress_static(x, n, eb, small, 64, res, g)
    assert nz.read_result(res)["status"] == nz.ERR_CAPACITY and nz.read_result(res)["bytes"] == 0
    big_n = 200 << 20
    assert nz.nz_workspace_bytes(big_n, nz.make_opts(chunk_elems=262144)) > nz.nz_static_scratch_bytes()
    assert nz.nz_compress_static(x, big_n, eb, out, sess.cap, res, nz.make_opts(chunk_elems=262144)) == nz.ERR_INVALID
    torch.cuda.synchronize()
