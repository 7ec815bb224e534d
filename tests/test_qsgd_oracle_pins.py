"""Pins for the QSGD part of the CPU oracle (oracle/qsgd_oracle.c): closed forms, library routines, brute force on
tiny inputs, the invariants and the expectation that Appendix B of the paper states, Monte Carlo checks of the
probabilities.  No GPU."""
import math

import numpy as np
import pytest

import oracle as ora
from tests.conftest import read_golden

RNG = np.random.default_rng(18100529)


def _gauss(d, scale=1e-2):
    return (RNG.standard_normal(d) * scale).astype(np.float32)


# ------------------------------------------------------------------ norms

def test_norms_closed_forms_and_library():
    assert ora.qsgd_norm_f64(np.array([3.0, -4.0], np.float32), ora.QSGD_L2) == 5.0
    assert ora.qsgd_norm_f64(np.array([3.0, -4.0], np.float32), ora.QSGD_MAX) == 4.0
    assert ora.qsgd_norm_f64(np.ones(1 << 16, np.float32), ora.QSGD_L2) == 256.0          # sqrt(k) for k ones
    assert ora.qsgd_norm_f64(np.full(49, -2.0, np.float32), ora.QSGD_L2) == 14.0
    assert ora.qsgd_norm_f64(np.zeros(10, np.float32), ora.QSGD_L2) == 0.0
    g = _gauss(100_003)
    ref = np.linalg.norm(g.astype(np.float64))
    assert abs(ora.qsgd_norm_f64(g, ora.QSGD_L2) - ref) <= 1e-12 * ref
    assert ora.qsgd_norm_f64(g, ora.QSGD_MAX) == float(np.abs(g).max())
    # L1 or a missing square root would fail the 3-4-5 case; a signed maximum fails this one
    assert ora.qsgd_norm_f64(np.array([1.0, -7.0, 2.0], np.float32), ora.QSGD_MAX) == 7.0
    # NaN does not take part in the maximum; it poisons the Euclidean norm
    withnan = np.array([1.0, np.nan, -3.0], np.float32)
    assert ora.qsgd_norm_f64(withnan, ora.QSGD_MAX) == 3.0
    assert math.isnan(ora.qsgd_norm_f64(withnan, ora.QSGD_L2))


def test_norms_composite_rows_strides_and_bf16():
    M, d = 4, 1000
    buf = np.full((M, d + 13), 1e30, np.float32)              # huge pads: must not be read
    buf[:, :d] = RNG.standard_normal((M, d)).astype(np.float32)
    for kind, ref in ((ora.QSGD_L2, np.linalg.norm(buf[:, :d].astype(np.float64), axis=1)),
                      (ora.QSGD_MAX, np.abs(buf[:, :d]).max(axis=1))):
        got = ora.qsgd_norms(buf[:, :d], kind)
        assert got.dtype == np.float32 and np.array_equal(got, ref.astype(np.float32))
    bits = ora.f32_to_bf16(buf[:, :d].copy())
    wide = ora.bf16_to_f32(bits)
    assert np.array_equal(ora.qsgd_norms(bits, ora.QSGD_L2), np.linalg.norm(wide.astype(np.float64), axis=1).astype(np.float32))


# ------------------------------------------------------------------ the ternary choice

def test_quantize_brute_force_on_small_vectors():
    # written differently: python floats rounded through numpy float32 scalars, one element at a time
    for trial in range(50):
        d = int(RNG.integers(1, 40))
        g = _gauss(d, 1.0)
        g[RNG.random(d) < 0.2] = 0.0
        u = RNG.random(d).astype(np.float32)
        norm = np.float32(np.sqrt(np.sum(g.astype(np.float64) ** 2)))
        q = ora.qsgd_quantize_row(g, u, norm)
        for i in range(d):
            t = np.float32(u[i]) * np.float32(norm)               # one fp32 rounding
            expect = 0
            if t < abs(g[i]):
                expect = 1 if g[i] > 0 else -1
            assert q[i] == expect, (trial, i)


def test_quantize_extremes_of_the_uniform_draw():
    g = _gauss(5000, 1.0)
    g[::11] = 0.0
    norm2 = np.float32(ora.qsgd_norm_f64(g, ora.QSGD_L2))
    # u = 0: probability-one end; every non-zero component is kept with its sign, zeros stay zero
    q0 = ora.qsgd_quantize_row(g, np.zeros_like(g), norm2)
    assert np.array_equal(q0, np.sign(g).astype(np.int8))
    # u just below 1 with the max norm: only components of the largest magnitude survive
    normi = np.float32(ora.qsgd_norm_f64(g, ora.QSGD_MAX))
    u1 = np.full_like(g, np.nextafter(np.float32(1.0), np.float32(0.0)))
    q1 = ora.qsgd_quantize_row(g, u1, normi)
    top = np.abs(g) == normi
    assert np.array_equal(q1 != 0, top & (np.float32(u1[0]) * normi < np.abs(g)))
    assert (q1[~top] == 0).all()
    # with the L2 norm and d > 1 non-zero components nothing survives u -> 1
    assert (ora.qsgd_quantize_row(g, u1, norm2) == 0).all()
    # zero gradient: norm 0, nothing kept whatever u is
    z = np.zeros(100, np.float32)
    assert (ora.qsgd_quantize_row(z, RNG.random(100).astype(np.float32), 0.0) == 0).all()
    # NaN is never kept, an infinite component with an infinite norm is not kept either (Inf < Inf is false)
    s = np.array([np.nan, np.inf, -np.inf, 1.0], np.float32)
    assert (ora.qsgd_quantize_row(s, np.full(4, 0.5, np.float32), np.inf) == 0).all()


def test_max_qsgd_leaves_sign_vectors_unchanged_and_single_entries_alone():
    # Appendix B: 1-bit max QSGD leaves sign vectors invariant; a vector with a single non-zero entry keeps that
    # entry (as +-1) and nothing else
    s = np.where(RNG.random(3000) < 0.5, -1.0, 1.0).astype(np.float32)
    norm = np.float32(ora.qsgd_norm_f64(s, ora.QSGD_MAX))
    assert norm == 1.0
    for _ in range(5):
        q = ora.qsgd_quantize_row(s, RNG.random(3000).astype(np.float32), norm)
        assert np.array_equal(q, s.astype(np.int8))
    for kind in (ora.QSGD_MAX, ora.QSGD_L2):
        e = np.zeros(777, np.float32)
        e[123] = -0.037
        q = ora.qsgd_quantize_row(e, RNG.random(777).astype(np.float32), np.float32(ora.qsgd_norm_f64(e, kind)))
        assert q[123] == -1 and np.count_nonzero(q) == 1


def test_scale_invariance_of_the_codes():
    # the codes depend on g / ||g|| only: scaling g by a power of two scales the norm by it, the codes stay
    g = _gauss(4096)
    u = RNG.random(4096).astype(np.float32)
    for kind in (ora.QSGD_L2, ora.QSGD_MAX):
        n1 = np.float32(ora.qsgd_norm_f64(g, kind))
        n2 = np.float32(ora.qsgd_norm_f64(g * np.float32(64), kind))
        assert n2 == n1 * np.float32(64)
        assert np.array_equal(ora.qsgd_quantize_row(g, u, n1), ora.qsgd_quantize_row(g * np.float32(64), u, n2))
        # negating g negates the codes
        assert np.array_equal(ora.qsgd_quantize_row(-g, u, n1), -ora.qsgd_quantize_row(g, u, n1))


@pytest.mark.parametrize("kind", [ora.QSGD_L2, ora.QSGD_MAX])
def test_keep_probability_and_unbiasedness_monte_carlo(kind):
    # P[component i kept] = |g_i| / ||g||  and  E[||g|| q_i] = g_i  (the quantiser is unbiased)
    d, trials = 64, 20_000
    g = _gauss(d, 1.0)
    norm = np.float32(ora.qsgd_norm_f64(g, kind))
    kept = np.zeros(d)
    mean = np.zeros(d)
    for _ in range(trials):
        q = ora.qsgd_quantize_row(g, RNG.random(d).astype(np.float32), norm)
        kept += q != 0
        mean += q.astype(np.float64) * norm
    p = np.abs(g) / norm
    sigma = np.sqrt(p * (1 - p) / trials)
    assert (np.abs(kept / trials - p) <= 5 * sigma + 1e-9).all()
    assert (np.abs(mean / trials - g) <= 5 * sigma * norm + 1e-9).all()


def test_expected_number_of_nonzeros_is_l1_over_l2_and_at_most_sqrt_d(golden):
    # Appendix B: E[# non-zero] = ||g||_1 / ||g||_2 <= sqrt(d)
    scal, _ = golden("qsgd_bits_per_iteration.txt")
    d, trials = 10_000, 300
    g = _gauss(d)
    norm = np.float32(ora.qsgd_norm_f64(g, ora.QSGD_L2))
    expect = np.abs(g.astype(np.float64)).sum() / float(norm)
    assert expect <= d ** scal["l2_expected_nonzero_bound_exponent_of_d"]
    counts = [np.count_nonzero(ora.qsgd_quantize_row(g, RNG.random(d).astype(np.float32), norm)) for _ in range(trials)]
    p = np.abs(g) / norm
    sigma = math.sqrt((p * (1 - p)).sum() / trials)
    assert abs(np.mean(counts) - expect) <= 5 * sigma
    # the bound is attained when all magnitudes are equal: then E[#] = d |c| / (|c| sqrt(d)) = sqrt(d) exactly
    c = np.where(RNG.random(d) < 0.5, -0.25, 0.25).astype(np.float32)
    nc = np.float32(ora.qsgd_norm_f64(c, ora.QSGD_L2))
    assert nc == np.float32(0.25 * 100)
    counts = [np.count_nonzero(ora.qsgd_quantize_row(c, RNG.random(d).astype(np.float32), nc)) for _ in range(trials)]
    assert abs(np.mean(counts) - math.sqrt(d)) <= 5 * math.sqrt(d * 0.01 * 0.99 / trials)
    # bits for a vector sent as (index, sign) pairs stay below sqrt(d) (1 + log d) in expectation
    assert np.mean(counts) * (scal["l2_sign_bits_per_nonzero"] + math.log2(d)) <= math.sqrt(d) * (1 + math.log2(d)) * 1.05


# ------------------------------------------------------------------ message format

def test_pack_format_bit_by_bit_and_round_trip(golden):
    scal, _ = golden("qsgd_bits_per_iteration.txt")
    for d in (1, 5, 63, 64, 65, 130, 1000):
        q = RNG.integers(-1, 2, size=d).astype(np.int8)
        nz, sg = ora.qsgd_pack(q)
        # reference written differently: strings of '0'/'1', least significant bit first
        for plane, pred in ((nz, lambda c: c != 0), (sg, lambda c: c > 0)):
            bits = "".join("1" if pred(c) else "0" for c in q).ljust(64 * len(plane), "0")
            for w in range(len(plane)):
                assert int(plane[w]) == int(bits[64 * w:64 * w + 64][::-1], 2)
        assert np.array_equal(ora.qsgd_unpack(nz, sg, d), q)
        # numpy's bit unpacking agrees
        un = np.unpackbits(nz.view(np.uint8), bitorder="little")[:d]
        assert np.array_equal(un.astype(bool), q != 0)
        # two planes of one bit per coordinate: the 2 d bits of Appendix B (rounded up to whole words)
        assert (nz.size + sg.size) * 64 == scal["max_bits_per_coordinate_upper"] * 64 * ((d + 63) // 64)
    # a sign bit never appears without its nonzero bit
    q = RNG.integers(-1, 2, size=4096).astype(np.int8)
    nz, sg = ora.qsgd_pack(q)
    assert ((sg & ~nz) == 0).all()


# ------------------------------------------------------------------ server average and update

def test_average_exact_cases_and_float64():
    # M = 1: the average is the decoded vector itself
    q = RNG.integers(-1, 2, size=(1, 500)).astype(np.int8)
    assert np.array_equal(ora.qsgd_average(q, np.array([0.75], np.float32)), q[0].astype(np.float32) * np.float32(0.75))
    # power-of-two norms, M = 4: every partial sum is exact, so the result equals the exact average
    M, d = 4, 2000
    q = RNG.integers(-1, 2, size=(M, d)).astype(np.int8)
    norms = np.array([1.0, 0.5, 2.0, 0.25], np.float32)
    exact = (q.astype(np.float64) * norms[:, None]).sum(axis=0) / M
    assert np.array_equal(ora.qsgd_average(q, norms).astype(np.float64), exact)
    # a worker with norm 0 contributes nothing; a missing 1/M or a dropped worker would fail the exact case above
    # general norms: within fp32 rounding of the float64 evaluation
    M, d = 15, 5000
    q = RNG.integers(-1, 2, size=(M, d)).astype(np.int8)
    norms = (RNG.random(M) * 3 + 0.1).astype(np.float32)
    a32, a64 = ora.qsgd_average(q, norms), ora.qsgd_average_f64(q, norms)
    ref = (q.astype(np.float64) * norms.astype(np.float64)[:, None]).sum(axis=0) / M
    assert np.allclose(a64, ref, rtol=1e-14, atol=0)
    scale = np.abs(q.astype(np.float64) * norms[:, None]).sum(axis=0) / M
    assert (np.abs(a32 - ref) <= 1e-6 * scale + 1e-30).all()


def test_update_exact_and_bf16_rounding():
    avg = np.array([0.5, -0.25, 0.0, 2.0], np.float32)
    x = np.array([1.0, 1.0, 1.0, 1.0], np.float32)
    ora.qsgd_update(x, avg, 0.5)
    assert np.array_equal(x, np.array([0.75, 1.125, 1.0, 0.0], np.float32))      # x - lr * avg, exact here
    # bf16 weights: widened, updated, rounded to nearest even -- against torch's cast
    import torch
    xb = torch.randn(4096, generator=torch.Generator().manual_seed(4)).to(torch.bfloat16)
    bits = xb.view(torch.int16).numpy().view(np.uint16).copy()
    avg = _gauss(4096, 1.0)
    ref = (xb.to(torch.float32) - torch.from_numpy(avg) * 0.125).to(torch.bfloat16)   # lr = 2^-3: the product is exact
    ora.qsgd_update(bits, avg, 0.125)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))


def test_composites_equal_the_steps_and_respect_strides():
    M, d = 5, 333
    gbuf = np.full((M, d + 7), np.nan, np.float32)
    gbuf[:, :d] = RNG.standard_normal((M, d)).astype(np.float32)
    ubuf = np.full((M, d + 3), 0.0, np.float32)
    ubuf[:, :d] = RNG.random((M, d)).astype(np.float32)
    for kind in (ora.QSGD_L2, ora.QSGD_MAX):
        norms = ora.qsgd_norms(gbuf[:, :d], kind)
        nz, sg = ora.qsgd_quantize(gbuf[:, :d], ubuf[:, :d], norms)
        q = np.stack([ora.qsgd_quantize_row(gbuf[m, :d].copy(), ubuf[m, :d].copy(), norms[m]) for m in range(M)])
        for m in range(M):
            assert np.array_equal(ora.qsgd_unpack(nz[m], sg[m], d), q[m])
        x = _gauss(d, 0.02)
        x_ref = x.copy()
        avg = ora.qsgd_aggregate_apply(nz, sg, norms, d, x, 0.1)
        assert np.array_equal(avg, ora.qsgd_average(q, norms))
        assert np.array_equal(x, ora.qsgd_update(x_ref, avg, 0.1))
        # float64 restatement of the whole 1-way scheme
        dec = q.astype(np.float64) * norms.astype(np.float64)[:, None]
        assert np.allclose(avg, dec.mean(axis=0), rtol=1e-5, atol=1e-9)


def test_one_way_qsgd_sgd_descends_on_a_quadratic():
    # f(x) = |x|^2 / 2 with noisy gradients, M = 3 workers (the worker count of the paper's QSGD figure): plain SGD on
    # the averaged decoded gradients must descend for both quantisers (unbiasedness in action)
    scal, _ = read_golden("qsgd_bits_per_iteration.txt")
    M, d = int(scal["qsgd_figure_workers"]), 200
    for kind in (ora.QSGD_L2, ora.QSGD_MAX):
        x = RNG.standard_normal(d).astype(np.float32)
        start = float((x.astype(np.float64) ** 2).sum())
        for _ in range(400):
            g = (x[None, :] + 0.1 * RNG.standard_normal((M, d))).astype(np.float32)
            norms = ora.qsgd_norms(g, kind)
            nz, sg = ora.qsgd_quantize(g, RNG.random((M, d)).astype(np.float32), norms)
            ora.qsgd_aggregate_apply(nz, sg, norms, d, x, 0.05)
        assert float((x.astype(np.float64) ** 2).sum()) < 0.2 * start
