"""The entry point that allocates nothing (ccoll_szx_decompress_static) against ccoll_szx_decompress_async.

Two calls in a row through the C ABI, the second on a smaller input, so that whatever the first call left
in the library's static scratch array (chunk offsets, result and error words) must not leak into the second;
then an error case (the status must clear again afterwards) and the size limit."""
import numpy as np
import pytest

import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_static_decompress_matches_context_decompress():
    import paper_2304_03890_amd as pkg
    ctx = pkg.Context(0, reserve_n=1 << 22)
    try:
        big = workloads.vector_1d(5120 * 300 + 77)
        small = workloads.blob_field((8, 64, 96), seed=5).ravel()[: 5120 * 9 + 130]
        res = torch.full((2,), -99, dtype=torch.int64, device="cuda")
        for x, rel in ((big, 1e-3), (small, 1e-4)):
            n = x.size
            eb = float(workloads.abs_bound(x, rel))
            s = ctx.compress(dev(x), eb).clone()
            want = torch.empty(n, dtype=torch.float32, device="cuda")
            assert ctx.decompress_async(s, n, want) == 0
            st, _ = ctx.wait()
            assert st == 0
            got = torch.full((n + 64,), 7.0, dtype=torch.float32, device="cuda")
            res.fill_(-99)
            rc = pkg.decompress_static(s, n, got, res)
            assert rc == 0, rc
            torch.cuda.synchronize()
            assert res.tolist() == [0, 0], res.tolist()
            assert torch.equal(got[:n].view(torch.int32), want.view(torch.int32)), n
            assert bool((got[n:] == 7.0).all()), "wrote past the end of the output"
        # a corrupt stream is reported through the result words, and the next call is clean again
        bad = s.clone()
        bad[40] ^= 0x7f                                   # an entry of the front index
        res.fill_(-99)
        assert pkg.decompress_static(bad, n, got, res) == 0
        torch.cuda.synchronize()
        assert res.tolist() == [0, pkg.ECORRUPT], res.tolist()
        res.fill_(-99)
        assert pkg.decompress_static(s, n, got, res) == 0
        torch.cuda.synchronize()
        assert res.tolist() == [0, 0]
        assert torch.equal(got[:n].view(torch.int32), want.view(torch.int32))
        # truncated below the front index: also through the result words
        assert pkg.decompress_static(s, n, got, res, in_bytes=33) == 0
        torch.cuda.synchronize()
        assert res.tolist() == [0, pkg.ECORRUPT]
        # beyond the limit of the static scratch: refused before anything is enqueued
        assert pkg.decompress_static(s, pkg.STATIC_MAX_ELEMS + 1, got, res) == pkg.EINVAL
        assert pkg.decompress_static(s, n, got, None) == pkg.EINVAL
    finally:
        ctx.close()
