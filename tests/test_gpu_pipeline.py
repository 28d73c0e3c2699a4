"""PIPE-SZx on one GPU (paper Sec. III-E.2): one stream written piece by piece on one HIP stream while a second
HIP stream forwards and decodes the pieces that are final -- the overlap of compression, transfer and
decompression that the paper gets by polling MPI between chunks.  The stream that arrives equals the oracle's
byte for byte, every piece decodes to the oracle's floats before the stream is complete."""
import numpy as np
import pytest

import workloads
from oracle import ref

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("shape,piece_chunks", [((40, 64, 96), 12), ((96, 128, 160), 120), ((100, 128, 160), 1200)])
def test_pieces_overlap_with_forward_and_decode(shape, piece_chunks):
    import paper_2304_03890_amd as pkg
    x = workloads.blob_field(shape, seed=31).ravel()
    x = x[: x.size - 333]                                   # ragged last chunk and block
    n = x.size
    nchunks = -(-n // 5120)
    eb = float(workloads.abs_bound(x, 1e-3))
    want = ref.compress(x, eb)
    full = ref.decompress(want, n)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ca, cb = pkg.Context(0, stream=sa, reserve_n=n), pkg.Context(0, stream=sb, reserve_n=n)
    try:
        dx = dev(x)
        cap = pkg.max_compressed_bytes(n)
        sent = torch.zeros(cap, dtype=torch.uint8, device="cuda")
        recv = torch.zeros(cap, dtype=torch.uint8, device="cuda")
        y = torch.full((n,), 7.0, dtype=torch.float32, device="cuda")
        bounds = list(range(0, nchunks, piece_chunks)) + [nchunks]
        k = len(bounds) - 1
        prog = torch.zeros(k, 2, dtype=torch.int64, device="cuda")
        res_a = torch.full((k, 2), -9, dtype=torch.int64, device="cuda")
        res_b = torch.full((k, 2), -9, dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()
        with torch.cuda.stream(sa):
            ca.compress_begin(n, eb, sent)
        events = []
        for i in range(k):
            with torch.cuda.stream(sa):
                assert ca.compress_chunks_async(dx, bounds[i], bounds[i + 1], prog[i], res_a[i]) == 0
                ev = torch.cuda.Event(); ev.record(sa); events.append(ev)
            with torch.cuda.stream(sb):                      # the "transport" and the receiver
                sb.wait_event(events[i])
                assert pkg.forward_async(recv, sent, n, prog[i - 1] if i else None, prog[i], hip_stream=sb.cuda_stream) == 0
                # the receiver decodes what has arrived; it cannot know the byte count on the host without a
                # round trip, so it offers the whole buffer: only the entries and payloads below chunk_end are read
                assert cb.decompress_chunks_async(recv, cap, n, bounds[i], bounds[i + 1], y[bounds[i] * 5120:], res_b[i]) == 0
        torch.cuda.synchronize()
        pr = prog.cpu().numpy()
        assert pr[:, 0].tolist() == bounds[1:]
        assert int(pr[-1, 1]) == want.size and (np.diff(pr[:, 1]) > 0).all()
        assert (res_a.cpu().numpy()[:, 1] == 0).all() and (res_b.cpu().numpy()[:, 1] == 0).all()
        assert res_a.cpu().numpy()[:, 0].tolist() == pr[:, 1].tolist()
        assert np.array_equal(sent[: want.size].cpu().numpy(), want), "the stream written in pieces"
        assert np.array_equal(recv[: want.size].cpu().numpy(), want), "the stream that was forwarded"
        assert np.array_equal(y.cpu().numpy().view(np.uint32), full.view(np.uint32)), "floats decoded piece by piece"
        # the complete stream decodes as any other
        out = cb.decompress(recv[: want.size], n)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), full.view(np.uint32))
    finally:
        ca.close(); cb.close()


def test_piece_rules_and_partial_streams():
    import paper_2304_03890_amd as pkg
    x = workloads.vector_1d(5120 * 50 + 77)
    n = x.size
    eb = float(np.float32(1e-3))
    want = ref.compress(x, eb)
    full = ref.decompress(want, n)
    ctx = pkg.Context(0, reserve_n=n)
    try:
        dx = dev(x)
        out = torch.zeros(pkg.max_compressed_bytes(n), dtype=torch.uint8, device="cuda")
        assert ctx.compress_chunks_async(dx, 0, 12) == pkg.EINVAL            # no stream begun
        ctx.compress_begin(n, eb, out)
        assert ctx.compress_chunks_async(dx, 0, 13) == pkg.EINVAL            # a piece ends at a multiple of 12 chunks
        assert ctx.compress_chunks_async(dx, 12, 24) == pkg.EINVAL           # pieces come in order
        assert ctx.compress_chunks_async(dx, 0, 24) == 0
        assert ctx.compress_chunks_async(dx, 24, 52) == pkg.EINVAL           # beyond the last chunk
        st, nb = ctx.wait()
        assert st == 0
        # what exists of the stream after the first piece: header with a total of 0, 24 index entries, 24 payloads
        part = out.cpu().numpy()
        idx = want[32:32 + 4 * 51].view(np.uint32)
        upto = 32 + 4 * 51 + int(idx[:24].sum())
        assert nb == upto
        assert np.array_equal(part[32:32 + 4 * 24], want[32:32 + 4 * 24]) and np.array_equal(part[32 + 4 * 51:upto], want[32 + 4 * 51:upto])
        assert part[24:32].view(np.uint64)[0] == 0
        y = torch.zeros(5120 * 24, dtype=torch.float32, device="cuda")
        assert ctx.decompress_chunks_async(out, upto, n, 0, 24, y) == 0
        st, _ = ctx.wait(); assert st == 0
        assert np.array_equal(y.cpu().numpy().view(np.uint32), full[:5120 * 24].view(np.uint32))
        assert ctx.decompress_chunks_async(out, upto - 4, n, 0, 24, y) == 0    # the last payload is not all there
        st, _ = ctx.wait(); assert st == pkg.ECORRUPT
        with pytest.raises(pkg.CcollError) as e:                                # the open stream is not a complete stream
            ctx.decompress(out[:upto], n)
        assert e.value.code == pkg.ECORRUPT
        assert ctx.compress_chunks_async(dx, 24, 51) == 0                       # the decode calls did not disturb the open stream
        st, nb = ctx.wait()
        assert st == 0 and nb == want.size
        assert np.array_equal(out[:nb].cpu().numpy(), want)
        assert ctx.compress_chunks_async(dx, 51, 51) == pkg.EINVAL              # the stream is complete
        # a compress call in between ends the open stream
        ctx.compress_begin(n, eb, out)
        assert ctx.compress_chunks_async(dx, 0, 12) == 0
        ctx.compress(dx[:5120], eb)
        assert ctx.compress_chunks_async(dx, 12, 24) == pkg.EINVAL
    finally:
        ctx.close()
