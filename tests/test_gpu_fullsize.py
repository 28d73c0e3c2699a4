"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py times: whole streams
against the CPU oracle byte for byte (the oracle codes 2^27 values in about a second), ranges and reduce
chains against the oracle and against the properties that hold at any size."""
import numpy as np
import pytest

import workloads
from oracle import ref

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2304_03890_amd as pkg
    c = pkg.Context(0, reserve_n=1 << 28)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def same_bytes(got, want, tag):
    assert got.size == want.size, (tag, got.size, want.size)
    if not np.array_equal(got, want):
        bad = np.nonzero(got != want)[0]
        raise AssertionError((tag, "first differing byte", int(bad[0]), "of", got.size))


@pytest.fixture(scope="module")
def field512():
    return workloads.blob_field((512, 512, 512))


@pytest.mark.parametrize("rel", [1e-2, 1e-3, 1e-4])
def test_field512_streams_match_oracle(ctx, field512, rel):
    """Workload 1 (the bench point is rel 1e-3): 26,215 chunks, four tiles of the index scan."""
    x = field512
    eb = float(workloads.abs_bound(x, rel))
    want = ref.compress(x, eb)
    dx = dev(x)
    got = ctx.compress(dx, eb)
    same_bytes(got.cpu().numpy(), want, f"compress rel={rel}")
    y = ctx.decompress(got, x.size)
    y_want = ref.decompress(want, x.size)
    assert torch.equal(y.view(torch.int32), dev(y_want).view(torch.int32)), f"decompress rel={rel}"
    err = (y.double() - dx.double()).abs().max().item()
    assert err <= float(np.float64(np.float32(eb))), (rel, err, eb)
    del y, y_want
    # reduce step with a second field: bytes against the oracle
    local = np.roll(x, 1)
    r_want = ref.reduce_step(local, want, eb)
    r_got = ctx.reduce_step(dev(local), got, eb)
    same_bytes(r_got.cpu().numpy(), r_want, f"reduce_step rel={rel}")


def test_ring_chunk_chain(ctx):
    """Workload 2 at its real shape: the chunk one rank owns after the reduce-scatter of P = 8 ranks,
    n = 143,667,240 / 8 = 17,958,405 values (last block 5 elements), abs eb 1e-5: one compress and seven
    reduce steps.  Every step's stream equals the oracle's; the result stays within P eb (+ the float32
    rounding of the seven adds) of the float64 sum (Eq. 2; worst case of Theorem 1's setting)."""
    n, P, eb = 143_667_240 // 8, 8, float(np.float32(1e-5))
    parts = [workloads.gradient_like(n, seed=workloads.SEED_GRAD + r) for r in range(P)]
    stream_ref = ref.compress(parts[0], eb)
    stream = ctx.compress(dev(parts[0]), eb)
    same_bytes(stream.cpu().numpy(), stream_ref, "ring round 0")
    for r in range(1, P):
        stream_ref = ref.reduce_step(parts[r], stream_ref, eb)
        stream = ctx.reduce_step(dev(parts[r]), stream, eb)
        same_bytes(stream.cpu().numpy(), stream_ref, f"ring round {r}")
    y = ctx.decompress(stream, n).cpu().numpy().astype(np.float64)
    exact = np.zeros(n, np.float64)
    for p in parts:
        exact += p
    mag = np.zeros(n, np.float64)
    for p in parts:
        mag += np.abs(p)
    slack = P * np.float64(eb) + P * mag * 2.0 ** -23 + P * np.float64(eb) * 2.0 ** -20
    assert (np.abs(y - exact) <= slack).all()


def test_bcast_field_ranges(ctx):
    """Workload 3: one 2^28-value field compressed once, decoded as 64 ranges of 2^22 values that start in
    the middle of chunks (32,768 blocks per range, 40 per chunk).  The stream and the whole decode equal the
    oracle's, every range equals its slice of that decode, and a sample of ranges equals the oracle's range
    decode."""
    x = workloads.bcast_field()
    n = x.size
    eb = float(workloads.abs_bound(x, 1e-3))
    want = ref.compress(x, eb)
    got = ctx.compress(dev(x), eb)
    same_bytes(got.cpu().numpy(), want, "bcast field stream")
    full = ctx.decompress(got, n)
    full_want = ref.decompress(want, n)
    assert torch.equal(full.view(torch.int32), dev(full_want).view(torch.int32)), "whole decode"
    del full_want
    cnt = n // 64
    for j in range(64):
        part = ctx.decompress_range(got, n, j * cnt, cnt)
        assert torch.equal(part.view(torch.int32), full[j * cnt:(j + 1) * cnt].view(torch.int32)), j
    for j in (0, 17, 63):
        r_want = ref.decompress_range(want, j * cnt, cnt)
        assert np.array_equal(full[j * cnt:(j + 1) * cnt].cpu().numpy().view(np.uint32), r_want.view(np.uint32)), j
    err = (full.double() - dev(x).double()).abs().max().item()
    assert err <= float(np.float64(np.float32(eb)))


@pytest.mark.parametrize("noise", [0.0, 0.25, 0.5, 1.0])
def test_sweep_points_match_oracle(ctx, noise):
    """Workload 4, all 20 points of the sweep (4 noise fractions x 5 bounds): from nearly all-constant blocks to
    white noise under a bound so tight that every block is stored raw and the chunks are larger than the
    coder's LDS stage (their bodies pass through the wavefront's spill slot).  Streams and decoded floats
    equal the oracle's; at two bounds per field also the reduce step with a shifted copy of the field."""
    x = workloads.sweep_mix(noise)
    dx = dev(x)
    for rel in (1e-2, 1e-3, 1e-4, 1e-5, 1e-6):
        eb = float(workloads.abs_bound(x, rel))
        want = ref.compress(x, eb)
        got = ctx.compress(dx, eb)
        same_bytes(got.cpu().numpy(), want, f"sweep noise={noise} rel={rel}")
        y = ctx.decompress(got, x.size)
        y_want = ref.decompress(want, x.size)
        assert torch.equal(y.view(torch.int32), dev(y_want).view(torch.int32)), (noise, rel)
        del y, y_want
        if rel in (1e-3, 1e-5):
            local = np.roll(x, 3)
            r_want = ref.reduce_step(local, want, eb)
            r_got = ctx.reduce_step(dev(local), got, eb)
            same_bytes(r_got.cpu().numpy(), r_want, f"sweep reduce noise={noise} rel={rel}")


def test_more_than_2_to_30_values(ctx):
    """The documented limit is n <= 2^31: one stream of 2^30 + 3 chunks + 77 values (4.3 GB of floats, 209,719
    chunks, 26 tiles of the index scan, offsets beyond 2^32 in a noisy part) against the oracle: stream bytes,
    decoded floats of both ends and of a range across the 2^32-byte mark of the input."""
    n = (1 << 30) + 5120 * 3 + 77
    base = workloads.vector_1d(1 << 22)
    noisy = (base + np.random.default_rng(3).standard_normal(base.size).astype(np.float32) * 0.05).astype(np.float32)
    x = np.empty(n, np.float32)
    for i0 in range(0, n, base.size):                      # smooth and noisy pieces in turns: CR about 1.65
        m = min(base.size, n - i0)
        x[i0:i0 + m] = (noisy if (i0 // base.size) % 2 else base)[:m]
    eb = float(workloads.abs_bound(base, 1e-5))
    ctx.reserve(n)
    dx = dev(x)
    got = ctx.compress(dx, eb)
    want = ref.compress(x, eb)
    assert got.numel() == want.size
    assert got.numel() > (1 << 31), "the stream should be longer than 2^31 bytes for this test to mean much"
    step = 1 << 28
    for o in range(0, want.size, step):                    # compare on the device, piece by piece
        assert torch.equal(got[o:o + step], dev(want[o:o + step])), ("stream bytes from", o)
    y = ctx.decompress(got, n)
    err = 0.0
    for o in range(0, n, step):
        err = max(err, (y[o:o + step].double() - dx[o:o + step].double()).abs().max().item())
    assert err <= float(np.float64(np.float32(eb)))
    for first, count in ((0, 5120 * 2 + 128), (n - 5120 - 77, 5120 + 77), ((1 << 30) - 128 * 50, 128 * 100)):
        part = ref.decompress_range(want, first, count)
        assert np.array_equal(y[first:first + count].cpu().numpy().view(np.uint32), part.view(np.uint32)), first
        r = ctx.decompress_range(got, n, first, count)
        assert np.array_equal(r.cpu().numpy().view(np.uint32), part.view(np.uint32)), first
