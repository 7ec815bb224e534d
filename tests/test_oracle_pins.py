"""Pins for the CPU oracle: everything here runs without a GPU and checks oracle/ against
things that are NOT the oracle -- brute force written differently, closed forms, invariants,
library routines (numpy bit unpacking, torch's bf16 cast, scipy's binomial), and the values the
paper prints (tests/golden/).  A dropped term, wrong sign, wrong bit index or transposed operand
in the oracle fails at least one of them."""
import math

import numpy as np
import pytest
import scipy.integrate
import scipy.stats
import torch

import oracle as ora
import workloads as wl
from tests.conftest import read_golden

RNG = np.random.default_rng(20181005)


# ------------------------------------------------------------------ sign + pack

def _bitstring_reference(x):
    """Independent statement of the message format: a string of '1'/'0', entry j at position j,
    cut into 64-character groups, each group read as a little-endian binary number."""
    chars = ["1" if (v >= 0) else "0" for v in x.tolist()]      # python float comparison
    while len(chars) % 64:
        chars.append("0")
    words = []
    for w in range(len(chars) // 64):
        grp = chars[64 * w: 64 * w + 64]
        words.append(int("".join(reversed(grp)), 2))
    return np.array(words, dtype=np.uint64)


@pytest.mark.parametrize("d", list(range(1, 200, 7)) + [63, 64, 65, 127, 128, 129, 200])
def test_sign_pack_bruteforce_small(d):
    x = RNG.standard_normal(d).astype(np.float32)
    x[RNG.integers(0, d, size=max(1, d // 10))] = 0.0
    got = ora.sign_pack(x[None, :])[0]
    assert np.array_equal(got, _bitstring_reference(x))


def test_sign_special_values():
    x = wl.special_values_f32()
    #              +0 -0 +den -den +min -min +1 -1 +inf -inf nan +big -big
    expected = [1, 1, 1, -1, 1, -1, 1, -1, 1, -1, -1, 1, -1]
    assert ora.sign_f32(x).tolist() == expected
    word = int(ora.sign_pack(x[None, :])[0, 0])
    assert word == sum(1 << i for i, s in enumerate(expected) if s > 0)


@pytest.mark.parametrize("d", list(range(1, 301)) + [65535, 65536, 65537])
def test_pack_unpack_roundtrip_and_padding(d):
    s = RNG.choice(np.array([-1, 1], dtype=np.int8), size=d)
    w = ora.pack_signs(s)
    assert w.size == (d + 63) // 64
    assert np.array_equal(ora.unpack_signs(w, d), s)
    # independent unpack through numpy's bit routines
    bits = np.unpackbits(w.view(np.uint8), bitorder="little")
    assert np.array_equal(bits[:d].astype(np.int8) * 2 - 1, s)
    assert not bits[d:].any(), "padding bits of the last word must be zero"


def test_sign_is_scale_invariant_and_negation_complements():
    # sign(v (x) g) = sign(v) (x) sign(g): a positive rescale changes nothing, a negative one
    # complements every bit whose entry is nonzero (proof of Theorem 2, first display).
    d = 1000
    x = RNG.standard_normal(d).astype(np.float32)
    base = ora.sign_pack(x[None, :])[0]
    for k in (-20, -3, 5, 30):
        assert np.array_equal(ora.sign_pack((x * np.float32(2.0 ** k))[None, :])[0], base)
    neg = ora.sign_pack((-x)[None, :])[0]
    mask = ora.pack_signs(np.ones(d, np.int8))          # valid-bit mask
    assert np.array_equal(neg, (~base) & mask)
    x[::5] = 0.0                                         # zeros keep +1 on both sides
    a, b = ora.sign_f32(x), ora.sign_f32(-x)
    assert np.array_equal(a[x != 0], -b[x != 0]) and (a[x == 0] == 1).all() and (b[x == 0] == 1).all()


def test_sign_pack_bf16_matches_torch_cast():
    x = torch.randn(3, 777, generator=torch.Generator().manual_seed(3)).to(torch.bfloat16)
    bits = wl.to_numpy(x)
    got = ora.sign_pack(bits)
    ref = ora.sign_pack(x.to(torch.float32).numpy())
    assert np.array_equal(got, ref)
    assert np.array_equal(ora.bf16_to_f32(bits), x.to(torch.float32).numpy())


def test_sign_pack_respects_row_strides():
    M, d = 4, 130
    buf = RNG.standard_normal((M, 160)).astype(np.float32)
    out = np.full((M, 5), np.uint64(0xFFFFFFFFFFFFFFFF))
    ora.sign_pack(buf[:, :d], signs=out[:, :3])
    for m in range(M):
        assert np.array_equal(out[m, :3], _bitstring_reference(buf[m, :d]))
    assert (out[:, 3:] == np.uint64(0xFFFFFFFFFFFFFFFF)).all()


# ------------------------------------------------------------------ momentum

def test_momentum_closed_form_constant_gradient():
    # v_0 = 0 and a constant gradient g give v_k = (1 - beta^k) g (geometric series).
    scal, _ = read_golden("algorithm1_defaults.txt")
    beta = scal["beta"]
    assert scal["initial_momentum"] == 0
    g = RNG.standard_normal(4096).astype(np.float32)
    v = np.zeros_like(g)
    b = np.float64(np.float32(beta))
    for k in range(1, 41):
        v64 = ora.momentum_f64(g, v, beta)                     # from the fp32 state before the step
        prev = (1.0 - b ** (k - 1)) * g.astype(np.float64)
        ora.momentum_f32(g, v, beta)
        exact = (1.0 - b ** k) * g.astype(np.float64)
        assert np.allclose(v, exact, rtol=1e-6, atol=0)
        assert np.allclose(v64, exact, rtol=2e-6, atol=0)
        assert np.allclose(v64 - b * prev, (1 - b) * g, rtol=1e-4)
    assert np.allclose(v, (1 - 0.9 ** 40) * g, rtol=1e-6)


def test_momentum_is_dampened_average_not_plain_accumulation():
    # One step from v = 1, g = 3, beta = 0.25:  (1-beta) g + beta v = 2.5   (plain v*beta+g would be 3.25)
    g = np.full(8, 3.0, np.float32)
    v = np.ones(8, np.float32)
    assert np.array_equal(ora.momentum_f32(g, v, 0.25), np.full(8, 2.5, np.float32))
    assert np.array_equal(ora.momentum_f64(g, np.ones(8, np.float32), 0.25), np.full(8, 2.5))
    # operands not swapped: beta multiplies v, (1-beta) multiplies g
    g = np.zeros(8, np.float32)
    v = np.full(8, 8.0, np.float32)
    assert np.array_equal(ora.momentum_f32(g, v, 0.25), np.full(8, 2.0, np.float32))


def test_momentum_beta_zero_is_the_gradient_and_scaling_is_exact():
    scal, _ = read_golden("algorithm1_defaults.txt")
    g = RNG.standard_normal(1000).astype(np.float32)
    v = RNG.standard_normal(1000).astype(np.float32)
    out = ora.momentum_f32(g, v.copy(), scal["beta_for_signsgd"])
    assert np.array_equal(out, g)
    a = ora.momentum_f32(g, v.copy(), 0.9)
    b = ora.momentum_f32(g * np.float32(1024), v * np.float32(1024), 0.9)
    assert np.array_equal(b, a * np.float32(1024))


def test_momentum_f32_close_to_f64():
    g = (RNG.standard_normal(100000) * 1e-2).astype(np.float32)
    v = (RNG.standard_normal(100000) * 3e-3).astype(np.float32)
    v64 = ora.momentum_f64(g, v, 0.9)
    v32 = ora.momentum_f32(g, v.copy(), 0.9)
    scale = np.abs(0.1 * g.astype(np.float64)) + np.abs(0.9 * v.astype(np.float64))
    assert (np.abs(v32 - v64) <= 1e-6 * scale).all()


# ------------------------------------------------------------------ vote

def _python_int_vote(patterns):
    """Vote by the definition with python integers: sign of the sum of +-1, zero -> +1."""
    out = []
    for col in patterns.T.tolist():
        tot = 0
        for s in col:
            tot += s
        out.append(1 if tot >= 0 else -1)
    return np.array(out, np.int8)


@pytest.mark.parametrize("M", list(range(1, 14)))
def test_vote_bruteforce_all_patterns(M):
    # every one of the 2^M sign patterns, one coordinate per pattern
    d = 1 << M
    idx = np.arange(d, dtype=np.int64)
    s = np.stack([(((idx >> m) & 1) * 2 - 1).astype(np.int8) for m in range(M)])
    V = ora.vote_sum(s)
    pop = np.array([bin(i).count("1") for i in range(d)])
    assert np.array_equal(V, 2 * pop - M)
    vote = ora.sign_i32(V)
    assert np.array_equal(vote, _python_int_vote(s))
    # the packed entry point agrees with the unpacked definition
    rows = np.stack([ora.pack_signs(s[m]) for m in range(M)])
    assert np.array_equal(ora.unpack_signs(ora.majority_vote(rows, d), d), vote)
    # threshold form: +1 iff at least ceil(M/2) workers say +1 (ties at even M go to +1)
    assert np.array_equal(vote > 0, pop >= (M + 1) // 2)


def test_vote_M1_identity_M3_textbook_majority():
    W = 50
    r = RNG.integers(0, 1 << 63, size=(3, W), dtype=np.int64).view(np.uint64) * np.uint64(2) + \
        RNG.integers(0, 2, size=(3, W)).astype(np.uint64)
    d = 64 * W
    assert np.array_equal(ora.majority_vote(r[:1], d), r[0])
    a, b, c = r
    assert np.array_equal(ora.majority_vote(r, d), (a & b) | (a & c) | (b & c))


@pytest.mark.parametrize("M", [2, 3, 4, 5, 6, 9, 12, 15, 16, 31, 100, 254, 255, 1023])
def test_vote_invariants(M):
    d = 3000 if M < 200 else 500
    s = RNG.choice(np.array([-1, 1], dtype=np.int8), size=(M, d), p=[0.45, 0.55])
    rows = np.stack([ora.pack_signs(s[m]) for m in range(M)])
    vote = ora.majority_vote(rows, d)
    v = ora.unpack_signs(vote, d)
    # against numpy popcount over workers
    pop = (s > 0).sum(axis=0)
    assert np.array_equal(v > 0, pop >= (M + 1) // 2)
    assert np.array_equal(v > 0, s.astype(np.int64).sum(axis=0) >= 0)
    # unanimity
    same = np.repeat(rows[:1], M, axis=0)
    assert np.array_equal(ora.majority_vote(same, d), rows[0])
    # permutation of workers
    assert np.array_equal(ora.majority_vote(rows[RNG.permutation(M)], d), vote)
    # negation: antisymmetric except exactly on ties
    mask = ora.pack_signs(np.ones(d, np.int8))
    vneg = ora.unpack_signs(ora.majority_vote((~rows) & mask, d), d)
    ties = (2 * pop == M)
    assert np.array_equal(vneg[~ties], -v[~ties])
    assert (vneg[ties] == 1).all() and (v[ties] == 1).all()
    if M % 2 == 1:
        assert not ties.any()
    # monotone: turning one worker's -1 into +1 never turns a +1 vote into -1
    s2 = s.copy()
    s2[RNG.integers(0, M)] = 1
    v2 = ora.sign_i32(ora.vote_sum(s2))
    assert (v2 >= v).all()
    # a +1 worker and a -1 worker added together cancel
    s3 = np.concatenate([s, np.ones((1, d), np.int8), -np.ones((1, d), np.int8)])
    assert np.array_equal(ora.sign_i32(ora.vote_sum(s3)), v)


def test_vote_ignores_row_padding_and_strides():
    M, d = 5, 100
    s = RNG.choice(np.array([-1, 1], dtype=np.int8), size=(M, d))
    buf = np.full((M, 4), np.uint64(0xFFFFFFFFFFFFFFFF))
    for m in range(M):
        buf[m, :2] = ora.pack_signs(s[m])
    buf[:, 1] |= np.uint64(0xFFFFFFF000000000)     # garbage in the padding bits (bits 36..63)
    vote = ora.majority_vote(buf[:, :2], d)
    assert np.array_equal(ora.unpack_signs(vote, d), ora.sign_i32(ora.vote_sum(s)))
    assert int(vote[1]) >> 36 == 0


# ------------------------------------------------------------------ adversaries (Definition 1, Theorem 2)

def _honest_and_adversary_sums(s, A):
    return s[A:].astype(np.int64).sum(axis=0), s[:A].astype(np.int64).sum(axis=0)


@pytest.mark.parametrize("M,A", [(15, 7), (7, 3), (27, 13), (9, 1)])
def test_margin_rule_and_inversion_characterisation(M, A):
    d = 20000
    g = (RNG.standard_normal(d) * 1e-3 + RNG.standard_normal((M, d)) * 1e-2).astype(np.float32)
    s = np.stack([ora.sign_f32(g[m]) for m in range(M)])
    VH, VA = _honest_and_adversary_sums(s, A)
    honest_vote = ora.sign_i32(ora.vote_sum(s))
    # arbitrary content in the adversarial rows: inverted, random, all +1, all -1
    for name in ("invert", "random", "plus", "minus"):
        t = s.copy()
        if name == "invert":
            t[:A] = -t[:A]
        elif name == "random":
            t[:A] = RNG.choice(np.array([-1, 1], dtype=np.int8), size=(A, d))
        else:
            t[:A] = 1 if name == "plus" else -1
        vote = ora.sign_i32(ora.vote_sum(t))
        safe = np.abs(VH) > A
        assert np.array_equal(vote[safe], np.sign(VH[safe])), name
        if name == "invert":
            differs = vote != honest_vote
            assert np.array_equal(differs, np.abs(VA) > np.abs(VH))
    # the whole-step entry point with worker_flip does the same inversion
    x = np.zeros(d, np.float32)
    flip = np.zeros(M, np.uint8)
    flip[:A] = 1
    vote_w, signs_w = ora.signum_step(g, None, 0.0, x, 1e-3, want_signs=True, worker_flip=flip)
    t = s.copy()
    t[:A] = -t[:A]
    assert np.array_equal(ora.unpack_signs(vote_w, d), ora.sign_i32(ora.vote_sum(t)))
    for m in range(M):
        assert np.array_equal(ora.unpack_signs(signs_w[m], d), t[m])


def _gaussian_vote_error(M, A, r, mode):
    """P[vote wrong] for signal N(0, r^2 sigma^2) and noise N(0, sigma^2): p = Phi(r|z|), honest
    workers Binomial(M-A, p), adversaries Binomial(A, 1-p) (invert) or Binomial(A, 1/2) (random);
    the vote is wrong when the number of correct bits is below M/2 (M odd)."""
    H = M - A
    kH, kA = np.arange(H + 1), np.arange(A + 1)

    def integrand(z):
        p = scipy.stats.norm.cdf(r * abs(z))
        q = {"invert": 1 - p, "random": 0.5, "none": p}[mode]
        pz = np.convolve(scipy.stats.binom.pmf(kH, H, p), scipy.stats.binom.pmf(kA, A, q))
        return pz[: (M + 1) // 2].sum() * scipy.stats.norm.pdf(z)

    return scipy.integrate.quad(integrand, -10, 10, limit=200)[0]


def test_vote_statistics_match_binomial_model():
    # low-SNR regime of the paper (Figure "SNR during training"): r = 0.1
    M, A, r, d = 15, 7, 0.1, 2_000_000
    scal, rows = read_golden("vote_binomial_model.txt")
    assert A / M < scal["max_adversary_fraction"]
    rng = np.random.default_rng(7)
    mu = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    g = (mu + rng.standard_normal((M, d)).astype(np.float32) * np.float32(1e-2)).astype(np.float32)
    x0 = np.zeros(d, np.float32)
    truth = ora.sign_f32(mu)
    vote_h, signs = ora.signum_step(g, None, 0.0, x0.copy(), 1e-4, want_signs=True)
    s0 = ora.unpack_signs(signs[0], d)
    tol = 5 * 0.5 / math.sqrt(d)
    # single worker: 1/2 - arctan(r)/pi
    assert abs((s0 != truth).mean() - (0.5 - math.atan(r) / math.pi)) < tol
    assert abs((ora.unpack_signs(vote_h, d) != truth).mean() - _gaussian_vote_error(M, 0, r, "none")) < tol
    flip = np.zeros(M, np.uint8)
    flip[:A] = 1
    vote_i, _ = ora.signum_step(g, None, 0.0, x0.copy(), 1e-4, worker_flip=flip)
    assert abs((ora.unpack_signs(vote_i, d) != truth).mean() - _gaussian_vote_error(M, A, r, "invert")) < tol
    # the model's mean and variance of Z (printed closed forms) at a fixed p
    for Mg, Ag, p, EZ, VZ in rows:
        Mg, Ag = int(Mg), int(Ag)
        n = 400_000
        correct = np.where(rng.random((Mg, n)) < p, 1, -1).astype(np.int8)   # +1 = correct bit
        correct[:Ag] = -correct[:Ag]                                          # inverting adversaries
        Z = (ora.vote_sum(correct) + Mg) // 2
        assert abs(Z.mean() - EZ) < 5 * math.sqrt(VZ / n)
        assert abs(Z.var() - VZ) < 0.03 * VZ
        fail = (ora.sign_i32(ora.vote_sum(correct)) < 0).mean()
        eps, alpha = p - 0.5, Ag / Mg
        cantelli = 1.0 / (1.0 + (EZ - Mg / 2) ** 2 / VZ)
        assert fail <= cantelli + 5 * 0.5 / math.sqrt(n)
        assert abs(EZ - (Mg / 2 + (1 - 2 * alpha) * Mg * eps)) < 1e-12


def test_lemma1_bound_holds_for_gaussian_noise():
    scal, rows = read_golden("lemma1_sign_failure_bound.txt")
    assert abs(scal["critical_snr"] - 2 / math.sqrt(3)) < 1e-15
    n = 1_000_000
    rng = np.random.default_rng(11)
    noise = rng.standard_normal(n).astype(np.float32)
    for S, bound in rows:
        formula = (2 / 9) / S ** 2 if S > 2 / math.sqrt(3) else 0.5 - S / (2 * math.sqrt(3))
        assert abs(formula - bound) < 1e-12 and bound <= 0.5
        if S == 0:
            continue
        err = (ora.sign_f32((np.float32(S) + noise).astype(np.float32)) < 0).mean()
        assert err <= bound + 5 * 0.5 / math.sqrt(n)
        assert abs(err - scipy.stats.norm.cdf(-S)) < 5 * 0.5 / math.sqrt(n)


def test_bimodal_worked_example_vote_follows_the_median_sign():
    scal, _ = read_golden("bimodal_example.txt")
    a, pa, b, pb = scal["value_a"], scal["prob_a"], scal["value_b"], scal["prob_b"]
    assert abs(a * pa + b * pb - scal["true_gradient_mean"]) < 1e-12
    n = 1_000_000
    rng = np.random.default_rng(5)
    for M in (1, 3, 15):
        g = np.where(rng.random((M, n)) < pa, a, b).astype(np.float32)
        assert abs(g.mean() - scal["true_gradient_mean"]) < 0.1
        x = np.zeros(n, np.float32)
        vote, _ = ora.signum_step(g, None, 0.0, x, 1.0)
        neg = (ora.unpack_signs(vote, n) < 0).mean()
        expect = scipy.stats.binom.cdf(M // 2, M, pa)      # at most M/2 workers drew the +50
        assert abs(neg - expect) < 5 * math.sqrt(max(expect * (1 - expect), 1e-6) / n)
        if M == 1:
            assert abs(neg - scal["prob_sign_negative"]) < 5 * 0.3 / math.sqrt(n)
        # the update moved every coordinate by exactly +-eta, against the voted sign
        assert np.array_equal(x, -ora.unpack_signs(vote, n).astype(np.float32))


# ------------------------------------------------------------------ update

def test_update_moves_by_exactly_eta_and_stays_on_lattice():
    d = 10000
    x0 = (RNG.standard_normal(d) * 0.02).astype(np.float32)
    vote = RNG.choice(np.array([-1, 1], dtype=np.int8), size=d)
    eta = np.float32(1e-4)
    x = ora.apply_f32(x0.copy(), vote, eta)
    expect = np.where(vote > 0, x0 - eta, x0 + eta).astype(np.float32)    # numpy fp32 add
    assert np.array_equal(x, expect)
    assert ((x < x0) == (vote > 0)).all()                                  # descends against the sign
    x64 = ora.apply_f64(x0, vote, eta)
    assert np.array_equal(x64, x0.astype(np.float64) - np.float64(eta) * vote)
    # k steps with a constant vote: x0 -+ k eta within k ulp
    xk = x0.copy()
    for _ in range(50):
        ora.apply_f32(xk, vote, eta)
    exact = x0.astype(np.float64) - 50 * np.float64(eta) * vote
    assert (np.abs(xk - exact) <= 50 * np.spacing(np.abs(x0) + 50 * eta)).all()


def test_update_with_weight_decay():
    x0 = np.array([0.5, -0.25, 2.0, -4.0], np.float32)
    vote = np.array([1, -1, -1, 1], np.int8)
    eta, lam = 0.125, 0.5            # exactly representable: every intermediate is exact
    x = ora.apply_f32(x0.copy(), vote, eta, lam)
    assert np.array_equal(x, np.array([0.5 - 0.125 * (1 + 0.25), -0.25 - 0.125 * (-1 - 0.125),
                                       2.0 - 0.125 * (-1 + 1.0), -4.0 - 0.125 * (1 - 2.0)], np.float32))
    assert np.array_equal(ora.apply_f64(x0, vote, eta, lam), x.astype(np.float64))
    xr = (RNG.standard_normal(5000)).astype(np.float32)
    vr = RNG.choice(np.array([-1, 1], dtype=np.int8), size=5000)
    a = ora.apply_f32(xr.copy(), vr, 1e-3, 1e-2)
    b = ora.apply_f64(xr, vr, 1e-3, 1e-2)
    assert np.allclose(a, b, rtol=1e-6, atol=1e-9)


def test_single_worker_reduces_to_plain_signsgd():
    # Theorem 1's iteration x_{k+1} = x_k - eta sign(g_k): M = 1, beta = 0, lambda = 0
    d = 5000
    g = RNG.standard_normal((1, d)).astype(np.float32)
    x0 = RNG.standard_normal(d).astype(np.float32)
    x = x0.copy()
    vote, signs = ora.signum_step(g, None, 0.0, x, 0.01, want_signs=True)
    assert np.array_equal(vote, signs[0])
    assert np.array_equal(x, (x0 - np.float32(0.01) * np.where(g[0] >= 0, 1, -1).astype(np.float32)))


def test_bf16_rounding_exhaustive_against_torch():
    # every bf16 bit pattern, both update directions; torch's cast is the independent RNE rounding
    bits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    xf = ora.bf16_to_f32(bits)
    tf = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(xf.view(np.uint32), tf.view(np.uint32))
    finite = np.isfinite(xf)
    for eta in (1e-5, 1e-3):
        for sgn in (1, -1):
            vote = np.full(bits.size, sgn, np.int8)
            got = ora.apply_bf16(bits.copy(), vote, eta)
            ref32 = (xf + np.float32(-sgn * np.float32(eta))).astype(np.float32)
            ref = torch.from_numpy(ref32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
            assert np.array_equal(got[finite], ref[finite])
            nan = np.isnan(xf)
            assert np.isnan(ora.bf16_to_f32(got[nan])).all()
    # random fp32 bit patterns through the rounding itself
    r = RNG.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    r = r[np.isfinite(r)]
    ref = torch.from_numpy(r.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ora.f32_to_bf16(r), ref)


def test_bf16_small_step_is_absorbed_for_large_weights():
    # with eta = 1e-5, |x| > 2^-8 has half-ulp > eta: the weight does not move
    x = torch.tensor([0.5, -0.5, 0.0059, 1e-4, -1e-4], dtype=torch.bfloat16)
    bits = wl.to_numpy(x)
    out = ora.apply_bf16(bits.copy(), np.ones(5, np.int8), 1e-5)
    assert np.array_equal(out[:3], bits[:3]) and (out[3:] != bits[3:]).all()


# ------------------------------------------------------------------ whole step

def _numpy_step(g, v, beta, x, lr, wd):
    """Algorithm 1 with numpy in float64, written independently of the C code."""
    b = np.float64(np.float32(beta))
    v_new = (1 - b) * g.astype(np.float64) + b * v.astype(np.float64)
    s = np.where(v_new >= 0, 1, -1)
    V = s.sum(axis=0)
    vote = np.where(V >= 0, 1, -1)
    x_new = x.astype(np.float64) - np.float64(np.float32(lr)) * (vote + np.float64(np.float32(wd)) * x)
    return v_new, s, vote, x_new


@pytest.mark.parametrize("M,d,beta,wd", [(3, 1000, 0.0, 0.0), (15, 5000, 0.9, 0.0), (6, 777, 0.5, 0.01),
                                          (31, 300, 0.99, 0.0)])
def test_whole_step_against_numpy_float64(M, d, beta, wd):
    g = (RNG.standard_normal(d) * 1e-3 + RNG.standard_normal((M, d)) * 1e-2).astype(np.float32)
    v = (RNG.standard_normal((M, d)) * 3e-3).astype(np.float32)
    x = (RNG.standard_normal(d) * 0.02).astype(np.float32)
    v_ref, s_ref, vote_ref, x_ref = _numpy_step(g, v, beta, x, 1e-4, wd)
    v_o, x_o = v.copy(), x.copy()
    vote, signs = ora.signum_step(g, v_o, beta, x_o, 1e-4, wd, want_signs=True)
    scale = np.abs((1 - beta) * g) + np.abs(beta * v) + 1e-30
    assert (np.abs(v_o - v_ref) <= 1e-6 * scale).all()
    decided = np.abs(v_ref) > 1e-6 * np.abs(v_ref).max()
    s_o = np.stack([ora.unpack_signs(signs[m], d) for m in range(M)])
    assert np.array_equal(s_o[decided], s_ref[decided])
    if decided.all():
        assert np.array_equal(ora.unpack_signs(vote, d), vote_ref)
        assert np.allclose(x_o, x_ref, rtol=1e-6, atol=1e-12)
    # the unfused entry points give the same bits and values as the whole step
    v_u, x_u = v.copy(), x.copy()
    signs_u = ora.signum_momentum_pack(g, v_u, beta)
    vote_u = ora.majority_vote(signs_u, d)
    ora.apply_sign_update(x_u, vote_u, 1e-4, wd)
    assert np.array_equal(signs_u, signs) and np.array_equal(vote_u, vote)
    assert np.array_equal(v_u, v_o) and np.array_equal(x_u, x_o)
    x_f = x.copy()
    vote_f = ora.vote_apply(signs_u, d, x_f, 1e-4, wd)
    assert np.array_equal(vote_f, vote) and np.array_equal(x_f, x_o)


@pytest.mark.parametrize("g_dtype", [np.float32, np.uint16])
def test_composites_respect_gradient_and_momentum_row_strides(g_dtype):
    # rows that sit in wider buffers (row stride != d, different for g, v and the packed signs): the result must
    # equal the float64 numpy restatement row by row, and nothing outside the rows may be read as data or written
    M, d, beta, lr = 5, 203, 0.75, 1e-3
    g32 = (RNG.standard_normal(d) * 1e-3 + RNG.standard_normal((M, d)) * 1e-2).astype(np.float32)
    if g_dtype == np.uint16:
        g_rows = ora.f32_to_bf16(g32)
        g32 = ora.bf16_to_f32(g_rows)
    else:
        g_rows = g32
    gbuf = np.full((M, d + 37), 0x7FC1 if g_dtype == np.uint16 else np.nan, dtype=g_dtype)   # NaN pads: must never be read
    gbuf[:, :d] = g_rows
    vbuf = np.full((M, d + 11), 123.0, np.float32)
    vbuf[:, :d] = (RNG.standard_normal((M, d)) * 3e-3).astype(np.float32)
    v0 = vbuf[:, :d].copy()
    x = (RNG.standard_normal(d) * 0.02).astype(np.float32)
    v_ref, s_ref, vote_ref, x_ref = _numpy_step(g32, v0, beta, x, lr, 0.0)
    decided = np.abs(v_ref) > 1e-6 * np.abs(v_ref).max()
    assert decided.all()

    W = ora.words_for(d)
    sbuf = np.full((M, W + 2), np.uint64(0xFFFFFFFFFFFFFFFF))
    ora.signum_momentum_pack(gbuf[:, :d], vbuf[:, :d], beta, signs=sbuf[:, :W])
    assert (vbuf[:, d:] == 123.0).all() and (sbuf[:, W:] == np.uint64(0xFFFFFFFFFFFFFFFF)).all()
    scale = np.abs((1 - beta) * g32) + np.abs(beta * v0)
    assert (np.abs(vbuf[:, :d] - v_ref) <= 1e-6 * scale).all()
    for m in range(M):
        assert np.array_equal(ora.unpack_signs(np.ascontiguousarray(sbuf[m, :W]), d), s_ref[m])

    vbuf2 = np.full((M, d + 5), -7.0, np.float32)
    vbuf2[:, :d] = v0
    x_o = x.copy()
    vote, signs = ora.signum_step(gbuf[:, :d], vbuf2[:, :d], beta, x_o, lr, want_signs=True)
    assert (vbuf2[:, d:] == -7.0).all()
    assert np.array_equal(vbuf2[:, :d], vbuf[:, :d])
    assert np.array_equal(signs, np.ascontiguousarray(sbuf[:, :W]))
    assert np.array_equal(ora.unpack_signs(vote, d), vote_ref)
    assert np.allclose(x_o, x_ref, rtol=1e-6, atol=1e-12)


def test_bf16_nan_keeps_sign_and_payload_and_gets_the_quiet_bit():
    # reading R5: a NaN is not rounded like a number (adding the rounding increment could carry into the
    # exponent and give Inf or flip the sign); its top 16 bits are kept and the quiet bit is set
    pat = np.array([0x7F800001, 0x7FC00000, 0xFF800001, 0xFFFFFFFF, 0x7FBFFFFF, 0x7F80FFFF, 0xFFC12345], np.uint32)
    out = ora.f32_to_bf16(pat.view(np.float32))
    assert np.array_equal(out, ((pat >> 16) | 0x40).astype(np.uint16))
    assert np.isnan(ora.bf16_to_f32(out)).all()
    assert np.array_equal(out >> 15, (pat >> 31).astype(np.uint16))           # sign kept
    # torch's cast agrees on NaN-ness (its payload convention is its own)
    t = torch.from_numpy(pat.view(np.float32).copy()).to(torch.bfloat16)
    assert torch.isnan(t).all()
    # and the infinities next to them are numbers: exact
    inf = np.array([np.inf, -np.inf], np.float32)
    assert np.array_equal(ora.f32_to_bf16(inf), np.array([0x7F80, 0xFF80], np.uint16))


def test_resume_is_bit_exact():
    M, d = 5, 2000
    mu = (RNG.standard_normal(d) * 1e-3).astype(np.float32)
    grads = [(mu + RNG.standard_normal((M, d)) * 1e-2).astype(np.float32) for _ in range(10)]
    x0 = (RNG.standard_normal(d) * 0.02).astype(np.float32)
    xa, va = x0.copy(), np.zeros((M, d), np.float32)
    for g in grads:
        ora.signum_step(g, va, 0.9, xa, 1e-4)
    xb, vb = x0.copy(), np.zeros((M, d), np.float32)
    for g in grads[:5]:
        ora.signum_step(g, vb, 0.9, xb, 1e-4)
    xb, vb = xb.copy(), vb.copy()                      # checkpoint = copies of x and v
    for g in grads[5:]:
        ora.signum_step(g, vb, 0.9, xb, 1e-4)
    assert np.array_equal(xa, xb) and np.array_equal(va, vb)
    # ten steps of +-eta keep every weight within 10 eta of its start, on the eta lattice
    steps = (xa.astype(np.float64) - x0) / 1e-4
    assert (np.abs(steps) <= 10 + 1e-3).all()
    assert np.allclose(steps, np.round(steps), atol=2e-2)
    assert (np.round(steps).astype(int) % 2 == 0).all()   # an even number of +-1 moves


def test_stress_input_generator_layout_and_statistics():
    # the pre-packed Bernoulli rows follow the message format, and the vote agrees with [p > 1/2]
    # at the rate the binomial model gives
    M, d = 255, 64 * 300 + 17
    rows_t, p_t = wl.bernoulli_packed_rows(M, d, seed=3, chunk_words=128)
    rows, p = wl.to_numpy(rows_t), p_t.numpy()
    assert rows.shape == (M, wl.words_for(d))
    s = np.stack([ora.unpack_signs(rows[m], d) for m in range(M)])
    mask = ora.pack_signs(np.ones(d, np.int8))
    assert ((rows & ~mask) == 0).all()
    dens = (s > 0).mean(axis=0)
    assert np.abs(dens - p).max() < 6 * 0.5 / math.sqrt(M)
    vote = ora.unpack_signs(ora.majority_vote(rows, d), d)
    agree = ((vote > 0) == (p > 0.5)).mean()
    expect = scipy.integrate.quad(lambda q: scipy.stats.binom.sf(127, 255, q) / 0.2, 0.5, 0.7)[0]
    assert abs(agree - expect) < 5 * math.sqrt(expect * (1 - expect) / d)


def test_communication_accounting():
    scal, _ = read_golden("communication_cost.txt")
    d, M = int(scal["resnet50_d"]), 15
    assert d == wl.RESNET50_D
    W = wl.words_for(d)
    assert W == scal["resnet50_words"] and d - 64 * (W - 1) == scal["resnet50_last_word_bits"]
    # one bit per coordinate per worker in each direction: 2 M d bits per iteration, and the
    # packed row is 32 times smaller than the fp32 gradient it stands for
    row_bits = ora.pack_signs(np.ones(64 * 1000, np.int8)).nbytes * 8
    assert row_bits == 64 * 1000
    assert (64 * 1000 * 32) / row_bits == scal["compression_vs_fp32"]
    assert scal["bits_per_iteration_factor"] * M * row_bits == 2 * M * 64 * 1000
