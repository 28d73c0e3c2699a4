"""Empirical check of the paper's error-propagation statements (Sec. III-B: Theorem 1, Corollaries 1 and 2,
Theorem 2) on the oracle, with synthetic data, for chains of P = 2 .. 8 ranks as the compressed ring
reduce-scatter builds them (Sec. III-A.2, Eq. 2: one compression per rank).

What is asserted is what holds for certain: every aggregated value lies within P eb of the exact aggregate
(plus the float32 rounding of the additions), and an average within eb.  The statistical statements are
measured and printed (run with -s), with loose sanity limits: the paper's model (normal single-step errors with
sigma = eb / 3) is an assumption about the compressor, not a property of this one, whose single-step error is
close to uniform.  tests/test_gpu_parity.py::test_error_propagation_on_the_device repeats the chains on the
GPU path."""
import numpy as np
import pytest

import workloads
from oracle import ref


def rank_fields(P, n, seed=77):
    rng = np.random.default_rng(seed)
    i = np.arange(n)
    return [(np.sin(i / (37.0 + 11 * r)) * (1 + 0.1 * r) + 0.25 * np.cos(i / (5.0 + r)) + 0.02 * rng.standard_normal(n)).astype(np.float32)
            for r in range(P)]


def chain_stats(parts, eb, op, compress, reduce_step, decompress):
    """For P = 1 .. len(parts): error of the chain's result against the exact float64 aggregate."""
    n = parts[0].size
    s = compress(parts[0], eb)
    exact = parts[0].astype(np.float64)
    out = [decompress(s, n).astype(np.float64) - exact]
    fn = {"sum": np.add, "max": np.maximum, "min": np.minimum}[op]
    for r in range(1, len(parts)):
        s = reduce_step(parts[r], s, eb, op)
        exact = fn(exact, parts[r].astype(np.float64))
        out.append(decompress(s, n).astype(np.float64) - exact)
    return out, exact


def report(parts, eb, errs_sum, errs_max, errs_min, exact_sum):
    sigma1 = errs_sum[0].std()
    lines = ["single step: sigma = %.4f eb (a normal error with eb = 3 sigma would have 0.3333; uniform rounding 0.2887 or less)" % (sigma1 / eb)]
    for P in range(2, len(parts) + 1):
        e = errs_sum[P - 1]
        th2 = 2.0 - (P + 2) / 2.0 ** P
        lines.append("P=%d  sum: std/(sqrt(P) sigma)=%.3f  inside +-(2/3)sqrt(P)eb: %.4f  max|e|/(P eb)=%.3f | avg: std/(sigma/sqrt(P))=%.3f | "
                     "max: var/sigma^2=%.3f (Thm 2: %.3f) max|e|/eb=%.3f | min: var/sigma^2=%.3f max|e|/eb=%.3f"
                     % (P, e.std() / (np.sqrt(P) * sigma1), float((np.abs(e) <= (2.0 / 3.0) * np.sqrt(P) * eb).mean()),
                        np.abs(e).max() / (P * eb), (e / P).std() / (sigma1 / np.sqrt(P)),
                        errs_max[P - 1].var() / sigma1 ** 2, th2, np.abs(errs_max[P - 1]).max() / eb,
                        errs_min[P - 1].var() / sigma1 ** 2, np.abs(errs_min[P - 1]).max() / eb))
    return lines


def check_bounds(parts, eb, errs, exact, op):
    for P in range(1, len(parts) + 1):
        e = np.abs(errs[P - 1])
        slack = P * np.float64(eb)
        if op == "sum":          # float32 rounding of the P - 1 additions
            mag = np.sum([np.abs(p.astype(np.float64)) for p in parts[:P]], axis=0)
            slack = slack + P * mag * 2.0 ** -23
        assert (e <= slack).all(), (op, P, float(e.max() / eb))


def test_sum_average_max_min_chains_on_the_oracle(capsys):
    P, n = 8, 5120 * 40 + 333
    eb = np.float32(2e-3)
    parts = rank_fields(P, n)
    ops = {}
    for op in ("sum", "max", "min"):
        errs, exact = chain_stats(parts, eb, op, ref.compress,
                                  lambda loc, s, e, o: ref.reduce_step(loc, s, e, op=o), ref.decompress)
        check_bounds(parts, eb, errs, exact, op)
        ops[op] = (errs, exact)
    errs_sum = ops["sum"][0]
    sigma1 = errs_sum[0].std()
    assert 0.15 * eb < sigma1 < 0.34 * eb                      # between "half the grid is unused" and the paper's eb / 3
    for k in range(2, P + 1):
        e = errs_sum[k - 1]
        # Theorem 1: the aggregated error grows like sqrt(P) sigma, not like P sigma (independent single-step errors)
        assert 0.6 < e.std() / (np.sqrt(k) * sigma1) < 1.4, k
        # Corollary 1: at least 95.44 % inside +-(2/3) sqrt(P) eb (this compressor's errors are lighter-tailed than normal)
        assert (np.abs(e) <= (2.0 / 3.0) * np.sqrt(k) * eb).mean() >= 0.9544, k
        # Corollary 2: an average is a sum divided once: within eb, spread sigma / sqrt(P)
        assert (np.abs(e / k) <= eb * (1 + 1e-6) + 1e-6).all()
        # Theorem 2's variance of max / min stays below 2 sigma^2 in the paper's model; here every step recompresses
        # the running result, so the spread may grow with P, but far more slowly than a sum's
        for op in ("max", "min"):
            assert ops[op][0][k - 1].var() < k * sigma1 ** 2 * 1.2, (op, k)
    with capsys.disabled():
        print()
        for line in report(parts, eb, errs_sum, ops["max"][0], ops["min"][0], ops["sum"][1]):
            print("   ", line)
