"""GPU parity: every entry point of libsignvote, called through its C ABI (via the thin binding),
against the CPU oracle on the same seeded inputs.  Bars: packed signs and votes bit-exact;
momentum and weights within 1e-6 relative of the float64 evaluation (and, because both sides fix
the same fp32 operation order, expected bit-identical to the fp32 oracle -- also asserted)."""
import numpy as np
import pytest
import torch

import oracle as ora
import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def sv():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_1810_05291_amd as sv_
    sv_.load_library()           # fails loudly when the HIP library is missing
    return sv_


def _log(*a):
    print(*a, flush=True)


def _strided(rows, cols, stride, dtype, fill=None):
    """[rows, cols] view of a [rows, stride] device buffer."""
    buf = torch.empty((rows, stride), dtype=dtype, device=DEV)
    if fill is not None:
        buf.fill_(fill)
    return buf, buf[:, :cols]


def _np_rows(t):
    """host copy of a (possibly strided) 2-D device view, contiguous; bf16 -> uint16 bits, int64 -> uint64"""
    return np.ascontiguousarray(wl.to_numpy(t.contiguous()))


RAGGED_D = [1, 3, 63, 64, 65, 255, 256, 257, 511, 1000, 4097, 65536, 100003]


# ------------------------------------------------------------------ sign_pack

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("d", RAGGED_D)
def test_sign_pack_ragged(sv, d, dtype):
    M = 3
    for stride in (d, ((d + 31) // 32) * 32, d + 1):
        _log(f"sign_pack d={d} dtype={dtype} stride={stride}")
        g = wl.gaussian((M, d), 1.0, seed=d, device=DEV)
        g[:, ::7] = 0.0
        buf, view = _strided(M, d, stride, dtype)
        view.copy_(g)
        W = sv.words_for(d)
        sbuf, sview = _strided(M, W, W + 3, torch.int64, fill=-1)
        sv.sign_pack(view, sview)
        torch.cuda.synchronize()
        ref = ora.sign_pack(_np_rows(view))
        assert np.array_equal(_np_rows(sview), ref)
        assert (sbuf[:, W:] == -1).all(), "wrote past the row"


def test_sign_pack_special_values(sv):
    x = torch.from_numpy(wl.special_values_f32()).to(DEV)[None, :]
    got = wl.to_numpy(sv.sign_pack(x))
    assert np.array_equal(got, ora.sign_pack(wl.special_values_f32()[None, :]))
    # scalar (unaligned) path sees the same values
    buf = torch.zeros(64, device=DEV)
    buf[1:1 + x.shape[1]] = x[0]
    got2 = wl.to_numpy(sv.sign_pack(buf[1:1 + x.shape[1]][None, :]))
    assert np.array_equal(got2, got)


# ------------------------------------------------------------------ momentum + pack

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,d,pad", [(1, 257, 0), (4, 1000, 0), (15, 100003, 0), (15, 100003, 29), (7, 65536, 0),
                                      (5, 12345, 3)])
def test_signum_momentum_pack(sv, M, d, pad, dtype):
    _log(f"momentum_pack M={M} d={d} pad={pad} dtype={dtype}")
    mu = wl.shared_mean(d, seed=1, device=DEV)
    _, v = _strided(M, d, d + pad, torch.float32, fill=0.0)
    v_ref = np.zeros((M, d), np.float32)
    for step in range(4):
        g = wl.worker_gradients(mu, M, step, base_seed=100, dtype=dtype, row_stride=d + pad)
        signs = sv.signum_momentum_pack(g, v, 0.9)
        torch.cuda.synchronize()
        g_h = _np_rows(g)
        g32 = g_h if dtype == torch.float32 else ora.bf16_to_f32(g_h)
        v64 = ora.momentum_f64(g32, v_ref, 0.9)
        scale = np.abs(0.1 * g32.astype(np.float64)) + np.abs(0.9 * v_ref.astype(np.float64))
        signs_ref = ora.signum_momentum_pack(g_h, v_ref, 0.9)
        v_gpu = _np_rows(v)
        assert (np.abs(v_gpu - v64) <= 1e-6 * scale + 1e-45).all()
        assert np.array_equal(v_gpu, v_ref)
        assert np.array_equal(_np_rows(signs), signs_ref)


# ------------------------------------------------------------------ majority vote

VOTE_M = [1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 254, 255, 256, 300, 1023]


@pytest.mark.parametrize("M", VOTE_M)
def test_majority_vote_random_rows(sv, M):
    for d, extra in ((64 * 700 + 17, 0), (64 * 513, 1), (200, 0), (64 * 129 + 63, 2)):
        W = sv.words_for(d)
        _log(f"majority_vote M={M} d={d} stride={W + extra}")
        buf = wl.random_words((M, W + extra), seed=M * 7 + d, device=DEV)
        rows = buf[:, :W]
        vote = sv.majority_vote(rows, d)
        torch.cuda.synchronize()
        ref = ora.majority_vote(_np_rows(rows), d)
        assert np.array_equal(wl.to_numpy(vote), ref)


@pytest.mark.parametrize("M", list(range(1, 13)))
def test_majority_vote_all_patterns(sv, M):
    # every one of the 2^M sign patterns, one coordinate each
    d = max(1 << M, 2)
    idx = np.arange(d, dtype=np.int64)
    s = np.stack([(((idx >> m) & 1) * 2 - 1).astype(np.int8) for m in range(M)])
    rows_h = np.stack([ora.pack_signs(s[m]) for m in range(M)])
    rows = torch.from_numpy(rows_h.view(np.int64)).to(DEV)
    vote = wl.to_numpy(sv.majority_vote(rows, d))
    assert np.array_equal(vote, ora.majority_vote(rows_h, d))


def test_majority_vote_ignores_and_clears_padding(sv):
    M, d = 5, 100
    rows = wl.random_words((M, 2), seed=9, device=DEV)
    vote = wl.to_numpy(sv.majority_vote(rows, d))
    rows_h = wl.to_numpy(rows).copy()
    assert np.array_equal(vote, ora.majority_vote(rows_h, d))
    assert int(vote[1]) >> 36 == 0
    rows_h[:, 1] ^= np.uint64(0xFFFFFFF000000000)                      # flip only padding bits
    vote2 = wl.to_numpy(sv.majority_vote(torch.from_numpy(rows_h.view(np.int64)).to(DEV), d))
    assert np.array_equal(vote, vote2)


# ------------------------------------------------------------------ apply / vote_apply

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("wd", [0.0, 0.01])
@pytest.mark.parametrize("d", RAGGED_D)
def test_apply_sign_update(sv, d, wd, dtype):
    lr = 1e-3 if dtype == torch.float32 else 1e-5
    for off in (0, 1):                                    # off = 1: base pointer not 16-byte aligned
        _log(f"apply d={d} wd={wd} dtype={dtype} off={off}")
        xbuf = wl.gaussian((d + 8,), 0.02, seed=d + 1, device=DEV).to(dtype)
        x = xbuf[off:off + d]
        x_h = wl.to_numpy(x.contiguous()).copy()
        x_before32 = x_h.copy() if dtype == torch.float32 else ora.bf16_to_f32(x_h)
        vote = wl.random_words((sv.words_for(d),), seed=d, device=DEV)
        sv.apply_sign_update(x, vote, lr, wd)
        torch.cuda.synchronize()
        vote_h = wl.to_numpy(vote)
        ora.apply_sign_update(x_h, vote_h, lr, wd)
        got = wl.to_numpy(x.contiguous())
        assert np.array_equal(got, x_h)
        x64 = ora.apply_f64(x_before32, ora.unpack_signs(vote_h, d), lr, wd)
        got32 = got if dtype == torch.float32 else ora.bf16_to_f32(got)
        # 1e-6 (fp32) or half a bf16 ulp, relative to the magnitude of the operands of the update
        tol = 1e-6 if dtype == torch.float32 else 2.0 ** -8
        scale = np.abs(x_before32.astype(np.float64)) * (1 + lr * wd) + lr
        assert (np.abs(got32 - x64) <= tol * scale).all()
        # guard elements around the view are untouched
        ref_buf = wl.gaussian((d + 8,), 0.02, seed=d + 1, device=DEV).to(dtype)
        assert torch.equal(xbuf[:off], ref_buf[:off]) and torch.equal(xbuf[off + d:], ref_buf[off + d:])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,d,extra,off", [(3, 65536, 0, 0), (15, 100003, 0, 0), (15, 64 * 1001, 1, 0),
                                            (31, 99999, 0, 1), (255, 20000, 0, 0), (6, 777, 0, 0),
                                            (16, 64 * 257 + 1, 1, 0), (1, 5, 0, 0)])
def test_vote_apply(sv, M, d, extra, off, dtype):
    _log(f"vote_apply M={M} d={d} extra={extra} off={off} dtype={dtype}")
    W = sv.words_for(d)
    rows = wl.random_words((M, W + extra), seed=M + d, device=DEV)[:, :W]
    for wd, want_vote in ((0.0, True), (0.02, False)):
        xbuf = wl.gaussian((d + 8,), 0.02, seed=5, device=DEV).to(dtype)
        x = xbuf[off:off + d]
        x_h = wl.to_numpy(x.contiguous()).copy()
        vote = torch.full((W,), -1, dtype=torch.int64, device=DEV) if want_vote else None
        lr = 1e-3 if dtype == torch.float32 else 1e-5
        sv.vote_apply(rows, d, x, lr, wd, vote_out=vote)
        torch.cuda.synchronize()
        vote_ref = ora.vote_apply(_np_rows(rows), d, x_h, lr, wd)
        assert np.array_equal(wl.to_numpy(x.contiguous()), x_h)
        if want_vote:
            assert np.array_equal(wl.to_numpy(vote), vote_ref)
        ref_buf = wl.gaussian((d + 8,), 0.02, seed=5, device=DEV).to(dtype)
        assert torch.equal(xbuf[:off], ref_buf[:off]) and torch.equal(xbuf[off + d:], ref_buf[off + d:])


# ------------------------------------------------------------------ whole fused step

def _step_case(sv, M, d, g_dtype, x_dtype, beta, wd, steps, pad=0, flip=None, momentum=True, lr=None,
               x_off=0, noise=1e-2, signal=1e-3):
    lr = lr if lr is not None else (1e-4 if x_dtype == torch.float32 else 1e-5)
    mu = wl.shared_mean(d, seed=11, device=DEV, std=signal)
    xbuf = wl.gaussian((d + 8,), 0.02, seed=12, device=DEV).to(x_dtype)
    x = xbuf[x_off:x_off + d]
    x_ref = wl.to_numpy(x.contiguous()).copy()
    v = v_ref = vbuf = None
    if momentum:
        vbuf, v = _strided(M, d, d + pad, torch.float32, fill=0.0)
        v_ref = np.zeros((M, d), np.float32)
    W = sv.words_for(d)
    near_zero = 0
    # Twin states.  A Signum call that gives room for the packed signs runs as two kernels (momentum + pack row by
    # row, then vote + update on the packed rows); without signs_out it is one kernel, in a lean instantiation
    # when no optional output or flip is asked for.  All three forms must agree bit for bit.
    x_lean = x.clone()
    v_lean = None if v is None else v.clone()
    x_one = x.clone()
    v_one = None if v is None else v.clone()
    for step in range(steps):
        g = wl.worker_gradients(mu, M, step, base_seed=500, noise_std=noise, dtype=g_dtype, row_stride=d + pad)
        vote_buf = torch.full((W + 2,), -1, dtype=torch.int64, device=DEV)
        vote = vote_buf[:W]
        signs_buf = torch.full((M, W + 1), -1, dtype=torch.int64, device=DEV)
        signs = signs_buf[:, :W]
        sv.signum_step(g, v, beta, x, lr, wd, vote_out=vote, signs_out=signs, worker_flip=flip)
        torch.cuda.synchronize()
        # nothing is written past the rows: guard words and pad columns keep their fill
        assert (vote_buf[W:] == -1).all() and (signs_buf[:, W:] == -1).all()
        if vbuf is not None and pad > 0:
            assert (vbuf[:, d:] == 0).all()
        g_h = _np_rows(g)
        v_prev = None if v_ref is None else v_ref.copy()
        vote_ref, signs_ref = ora.signum_step(g_h, v_ref, beta, x_ref, lr, wd, want_signs=True, worker_flip=flip)
        signs_gpu = _np_rows(signs)
        if momentum:
            g32 = g_h if g_dtype == torch.float32 else ora.bf16_to_f32(g_h)
            v64 = ora.momentum_f64(g32, v_prev, beta)
            v_gpu = _np_rows(v)
            scale = np.abs((1 - beta) * g32.astype(np.float64)) + np.abs(beta * v_prev.astype(np.float64))
            assert (np.abs(v_gpu - v64) <= 1e-6 * scale + 1e-45).all(), "momentum outside 1e-6 relative"
            # sign bits may differ only where |m| < 1e-6 max|m|; count them (expected 0)
            diff = signs_gpu != signs_ref
            if diff.any():
                tiny = np.abs(v64) < 1e-6 * np.abs(v64).max()
                bad = [ora.unpack_signs(signs_gpu[m], d) != ora.unpack_signs(signs_ref[m], d) for m in range(M)]
                bad = np.stack(bad)
                assert not (bad & ~tiny).any(), "sign differs on a decided coordinate"
                near_zero += int(bad.sum())
            assert np.array_equal(v_gpu, v_ref), "fp32 momentum not bit-identical to the fp32 oracle"
        assert np.array_equal(signs_gpu, signs_ref)
        assert np.array_equal(wl.to_numpy(vote), vote_ref)
        x_gpu = wl.to_numpy(x.contiguous())
        assert np.array_equal(x_gpu, x_ref)
        vote_one = torch.full((W + 2,), -1, dtype=torch.int64, device=DEV)
        sv.signum_step(g, v_one, beta, x_one, lr, wd, vote_out=vote_one[:W], worker_flip=flip)
        torch.cuda.synchronize()
        assert (vote_one[W:] == -1).all() and torch.equal(vote_one[:W], vote), "one-kernel form disagrees (vote)"
        assert torch.equal(x_one, x), "one-kernel form disagrees (weights)"
        assert v is None or torch.equal(v_one, v), "one-kernel form disagrees (momentum)"
        if flip is None:
            sv.signum_step(g, v_lean, beta, x_lean, lr, wd)
            torch.cuda.synchronize()
            assert torch.equal(x_lean, x), "form without optional outputs disagrees (weights)"
            assert v is None or torch.equal(v_lean, v), "form without optional outputs disagrees (momentum)"
    ref_buf = wl.gaussian((d + 8,), 0.02, seed=12, device=DEV).to(x_dtype)
    assert torch.equal(xbuf[:x_off], ref_buf[:x_off]) and torch.equal(xbuf[x_off + d:], ref_buf[x_off + d:])
    return near_zero


def test_step_tiny_config_signsgd(sv):
    # config 'tiny': d = 65,536, M = 3, plain signSGD, lr = 1e-3, one step -- fused and unfused
    g, x = wl.tiny_config(seed=0, device=DEV)
    M, d = g.shape
    x_ref = wl.to_numpy(x).copy()
    x_f = x.clone()
    vote = torch.empty((sv.words_for(d),), dtype=torch.int64, device=DEV)
    sv.signum_step(g, None, 0.0, x_f, 1e-3, vote_out=vote)
    x_u = x.clone()
    signs = sv.sign_pack(g)
    vote_u = sv.majority_vote(signs, d)
    sv.apply_sign_update(x_u, vote_u, 1e-3)
    x_v = x.clone()
    sv.vote_apply(signs, d, x_v, 1e-3)
    torch.cuda.synchronize()
    vote_ref, signs_ref = ora.signum_step(wl.to_numpy(g), None, 0.0, x_ref, 1e-3, want_signs=True)
    assert np.array_equal(wl.to_numpy(signs), signs_ref)
    assert np.array_equal(wl.to_numpy(vote), vote_ref) and np.array_equal(wl.to_numpy(vote_u), vote_ref)
    for t in (x_f, x_u, x_v):
        assert np.array_equal(wl.to_numpy(t), x_ref)
    x64 = ora.apply_f64(wl.to_numpy(x), ora.unpack_signs(vote_ref, d), 1e-3)
    assert (np.abs(wl.to_numpy(x_f) - x64) <= 1e-6 * (np.abs(wl.to_numpy(x)) + 1e-3)).all()


@pytest.mark.parametrize("M,d,pad,x_off", [(1, 1, 0, 0), (2, 64, 0, 0), (3, 257, 0, 0), (15, 100003, 0, 0),
                                            (15, 100003, 1, 0), (15, 100000, 0, 1), (31, 70001, 3, 0),
                                            (16, 4096, 0, 0), (40, 3000, 0, 0), (255, 4097, 0, 0),
                                            (1023, 2049, 0, 0), (1022, 700, 2, 1),
                                            # beyond 2^21 coordinates the one-kernel form holds 4 tiles per wave instead of 1
                                            (3, (1 << 21) + 4099, 0, 0), (5, (1 << 21) + 258, 1, 1)])
def test_step_signum_fp32(sv, M, d, pad, x_off):
    _log(f"signum_step fp32 M={M} d={d} pad={pad} x_off={x_off}")
    nz = _step_case(sv, M, d, torch.float32, torch.float32, 0.9, 0.0, steps=3, pad=pad, x_off=x_off)
    _log(f"  near-zero sign exceptions: {nz}")
    assert nz == 0


@pytest.mark.parametrize("g_dtype,x_dtype", [(torch.bfloat16, torch.bfloat16), (torch.bfloat16, torch.float32),
                                              (torch.float32, torch.bfloat16)])
@pytest.mark.parametrize("M,d,pad", [(31, 100003, 0), (31, 65536 + 8, 0), (5, 999, 5), (3, 8, 0), (3, (1 << 21) + 777, 0)])
def test_step_signum_mixed_dtypes(sv, M, d, pad, g_dtype, x_dtype):
    _log(f"signum_step M={M} d={d} pad={pad} g={g_dtype} x={x_dtype}")
    assert _step_case(sv, M, d, g_dtype, x_dtype, 0.9, 0.0, steps=2, pad=pad) == 0


def test_step_weight_decay_flip_and_no_momentum(sv):
    flip = [1, 0, 1, 0, 0, 1, 0]
    assert _step_case(sv, 7, 50001, torch.float32, torch.float32, 0.5, 0.01, steps=2, flip=flip) == 0
    assert _step_case(sv, 7, (1 << 21) + 50001, torch.float32, torch.float32, 0.5, 0.01, steps=2, flip=flip) == 0   # 4 tiles per wave
    assert _step_case(sv, 7, 50001, torch.float32, torch.float32, 0.0, 0.0, steps=1, flip=flip, momentum=False) == 0
    assert _step_case(sv, 6, 3001, torch.bfloat16, torch.bfloat16, 0.0, 0.001, steps=1, momentum=False) == 0
    # beta = 0 with a momentum buffer: v becomes the gradient
    assert _step_case(sv, 4, 3001, torch.float32, torch.float32, 0.0, 0.0, steps=2) == 0


def test_step_special_values_do_not_spread(sv):
    # an infinite / NaN gradient from one worker is one vote, nothing more (Section 1 on faulty workers)
    M, d = 5, 1024
    g = wl.gaussian((M, d), 1.0, seed=3, device=DEV)
    g[0, :256] = float("inf")
    g[0, 256:512] = float("-inf")
    g[0, 512:768] = float("nan")
    g[1, ::3] = 0.0
    g[2, ::5] = -0.0
    x = wl.gaussian((d,), 0.02, seed=4, device=DEV)
    v = torch.zeros((M, d), device=DEV)
    x_ref, v_ref = wl.to_numpy(x).copy(), np.zeros((M, d), np.float32)
    vote = torch.empty((sv.words_for(d),), dtype=torch.int64, device=DEV)
    signs = torch.empty((M, sv.words_for(d)), dtype=torch.int64, device=DEV)
    # the same state through the one-kernel forms (with and without the packed vote as output)
    x_one, v_one, x_lean, v_lean = x.clone(), v.clone(), x.clone(), v.clone()
    vote_one = torch.empty_like(vote)
    for _ in range(2):
        sv.signum_step(g, v, 0.9, x, 1e-3, vote_out=vote, signs_out=signs)          # two kernels
        sv.signum_step(g, v_one, 0.9, x_one, 1e-3, vote_out=vote_one)
        sv.signum_step(g, v_lean, 0.9, x_lean, 1e-3)
        torch.cuda.synchronize()
        vote_ref, signs_ref = ora.signum_step(wl.to_numpy(g), v_ref, 0.9, x_ref, 1e-3, want_signs=True)
        assert np.array_equal(wl.to_numpy(signs), signs_ref)
        assert np.array_equal(wl.to_numpy(vote), vote_ref) and torch.equal(vote_one, vote)
        assert np.array_equal(wl.to_numpy(x), x_ref) and torch.equal(x_one, x) and torch.equal(x_lean, x)
        nan = np.isnan(v_ref)                      # NaN payloads are not compared, NaN-ness is
        for v_form in (v, v_one, v_lean):
            v_gpu = wl.to_numpy(v_form)
            assert np.array_equal(np.isnan(v_gpu), nan) and np.array_equal(v_gpu[~nan], v_ref[~nan])
    assert np.isfinite(wl.to_numpy(x)).all()


def _bf16_tensor(bits):
    """device bf16 tensor from uint16 bit patterns"""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def _same_up_to_nan_payload_bf16(got, ref):
    nan_g, nan_r = np.isnan(ora.bf16_to_f32(got)), np.isnan(ora.bf16_to_f32(ref))
    return np.array_equal(nan_g, nan_r) and np.array_equal(got[~nan_r], ref[~nan_r])


def test_step_special_values_bf16(sv):
    # bf16 gradients AND bf16 weights holding +-Inf, NaN, +-0 and bf16 denormals: a faulty worker is one vote,
    # and a weight that is already Inf / NaN stays what IEEE arithmetic makes of it, identically on both sides
    M, d = 5, 2048
    rng = np.random.default_rng(5)
    g_bits = ora.f32_to_bf16((rng.standard_normal((M, d)) * 1e-2).astype(np.float32))
    g_bits[0, :256] = 0x7F80          # +Inf
    g_bits[0, 256:512] = 0xFF80       # -Inf
    g_bits[0, 512:768] = 0x7FC0       # NaN
    g_bits[3, 512:640] = 0xFFC1       # NaN with the sign bit set
    g_bits[1, ::3] = 0x0000           # +0
    g_bits[2, ::5] = 0x8000           # -0
    g_bits[4, 1024:1280] = 0x0001     # smallest positive bf16 denormal
    g_bits[4, 1280:1536] = 0x8001     # and its negative
    x_bits = ora.f32_to_bf16((rng.standard_normal(d) * 0.02).astype(np.float32))
    x_bits[100:110] = 0x7F80
    x_bits[110:120] = 0xFF80
    x_bits[120:130] = 0x7FC0
    x_bits[130:140] = 0x0000
    x_bits[140:150] = 0x8000
    x_bits[150:160] = 0x0001
    x_bits[160:170] = 0x7F7F          # largest finite bf16: the step must not overflow it by rounding
    for wd in (0.0, 0.01):
        g, x = _bf16_tensor(g_bits), _bf16_tensor(x_bits)
        v = torch.zeros((M, d), device=DEV)
        x_ref, v_ref = x_bits.copy(), np.zeros((M, d), np.float32)
        W = sv.words_for(d)
        vote = torch.empty((W,), dtype=torch.int64, device=DEV)
        signs = torch.empty((M, W), dtype=torch.int64, device=DEV)
        x_one, v_one, vote_one = _bf16_tensor(x_bits), torch.zeros((M, d), device=DEV), torch.empty_like(vote)
        for step in range(2):
            sv.signum_step(g, v, 0.9, x, 1e-3, wd, vote_out=vote, signs_out=signs)      # two kernels
            sv.signum_step(g, v_one, 0.9, x_one, 1e-3, wd, vote_out=vote_one)           # one kernel
            torch.cuda.synchronize()
            vote_ref, signs_ref = ora.signum_step(g_bits, v_ref, 0.9, x_ref, 1e-3, wd, want_signs=True)
            assert np.array_equal(wl.to_numpy(signs), signs_ref), f"signs, step {step}"
            assert np.array_equal(wl.to_numpy(vote), vote_ref) and torch.equal(vote_one, vote), f"vote, step {step}"
            assert _same_up_to_nan_payload_bf16(wl.to_numpy(x), x_ref), f"weights, step {step}"
            assert _same_up_to_nan_payload_bf16(wl.to_numpy(x_one), x_ref), f"weights of the one-kernel form, step {step}"
            nan = np.isnan(v_ref)
            for v_form in (v, v_one):
                v_gpu = wl.to_numpy(v_form)
                assert np.array_equal(np.isnan(v_gpu), nan) and np.array_equal(v_gpu[~nan], v_ref[~nan])
        # the unfused update from the same vote sees the same special weights
        x2 = _bf16_tensor(x_bits)
        x2_ref = x_bits.copy()
        sv.apply_sign_update(x2, vote, 1e-3, wd)
        torch.cuda.synchronize()
        ora.apply_sign_update(x2_ref, vote_ref, 1e-3, wd)
        assert _same_up_to_nan_payload_bf16(wl.to_numpy(x2), x2_ref)
        # fp32 weights with the same specials through the stand-alone update and the fused vote + update
        x32_h = ora.bf16_to_f32(x_bits)
        for fn in ("apply", "vote_apply"):
            x32 = torch.from_numpy(x32_h.copy()).to(DEV)
            x32_ref = x32_h.copy()
            if fn == "apply":
                sv.apply_sign_update(x32, vote, 1e-3, wd)
            else:
                sv.vote_apply(signs, d, x32, 1e-3, wd)
            torch.cuda.synchronize()
            ora.apply_sign_update(x32_ref, vote_ref, 1e-3, wd)
            got = wl.to_numpy(x32)
            nan = np.isnan(x32_ref)
            assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], x32_ref[~nan]), fn


@pytest.mark.parametrize("g_kind", ["f32", "bf16"])
def test_denormal_momentum_is_not_flushed(sv, g_kind):
    # gradients so small that (1-beta) g and fma(beta, v, .) are fp32 denormals, of both signs: the sign of a
    # denormal is data (a flushed negative denormal would read as -0 and vote +1).  Signs, the bits of v and the
    # vote must equal the oracle's; the oracle runs on an x86 host, which keeps denormals.
    M, d = 7, 70_003
    rng = np.random.default_rng(11)
    W = sv.words_for(d)
    v = torch.zeros((M, d), device=DEV)
    v_ref = np.zeros((M, d), np.float32)
    x = wl.gaussian((d,), 0.02, seed=3, device=DEV)
    x_ref = wl.to_numpy(x).copy()
    x_lean, v_lean = x.clone(), v.clone()
    seen_denormal = False
    for step in range(3):
        if g_kind == "f32":
            # magnitudes 1e-44 .. 1e-38: denormal or barely normal; products with 0.1 are all denormal
            mag = (10.0 ** rng.uniform(-44, -38, size=(M, d)))
            g_h = (np.where(rng.random((M, d)) < 0.5, -1.0, 1.0) * mag).astype(np.float32)
            g = torch.from_numpy(g_h).to(DEV)
        else:
            # bf16 denormals (exponent field 0, any mantissa) and the smallest normals, both signs
            g_h = (rng.integers(1, 0x0100, size=(M, d)).astype(np.uint16)
                   | (rng.integers(0, 2, size=(M, d)).astype(np.uint16) << 15))
            g = _bf16_tensor(g_h)
        assert np.array_equal(wl.to_numpy(g), g_h), "the device copy must hold the denormals"
        vote = torch.empty((W,), dtype=torch.int64, device=DEV)
        signs = torch.empty((M, W), dtype=torch.int64, device=DEV)
        sv.signum_step(g, v, 0.9, x, 1e-4, vote_out=vote, signs_out=signs)
        sv.signum_step(g, v_lean, 0.9, x_lean, 1e-4)                       # lean form
        torch.cuda.synchronize()
        vote_ref, signs_ref = ora.signum_step(g_h, v_ref, 0.9, x_ref, 1e-4, want_signs=True)
        tiny = np.finfo(np.float32).tiny
        frac = ((np.abs(v_ref) < tiny) & (v_ref != 0)).mean()
        seen_denormal |= frac > 0.5
        assert np.array_equal(wl.to_numpy(v), v_ref), f"momentum bits differ at step {step}"
        assert np.array_equal(wl.to_numpy(signs), signs_ref), f"signs differ at step {step}"
        assert np.array_equal(wl.to_numpy(vote), vote_ref), f"vote differs at step {step}"
        assert np.array_equal(wl.to_numpy(x), x_ref)
        assert torch.equal(v_lean, v) and torch.equal(x_lean, x)
        # and through the unfused momentum + pack entry point from the same state
        if step == 0:
            v2 = torch.zeros((M, d), device=DEV)
            s2 = sv.signum_momentum_pack(g, v2, 0.9)
            torch.cuda.synchronize()
            assert np.array_equal(wl.to_numpy(s2), signs_ref) and np.array_equal(wl.to_numpy(v2), v_ref)
    assert seen_denormal, "the test did not reach the denormal range"
    negative_denormals = int(((v_ref < 0) & (np.abs(v_ref) < np.finfo(np.float32).tiny)).sum())
    _log(f"denormal momentum ({g_kind}): {negative_denormals} negative denormal entries kept their sign")
    assert negative_denormals > 1000


# ------------------------------------------------------------------ multi-tensor step (pointer table)

def _ragged_sizes(rng, T):
    """Tensor sizes like a model's: biases below a wavefront, odd lengths, exact multiples of the 4096-coordinate
    unit and of the 256-coordinate tile, and a few large tensors that span many units."""
    fixed = [1, 2, 3, 5, 17, 63, 64, 65, 255, 256, 257, 1000, 4095, 4096, 4097, 8192, 12_289, 65_536, 100_003, 262_147]
    sizes = fixed + [int(rng.integers(1, 3000)) for _ in range(T - len(fixed))]
    rng.shuffle(sizes)
    return sizes


@pytest.mark.parametrize("two_kernels", [False, True])
@pytest.mark.parametrize("g_dtype,x_dtype,momentum", [(torch.float32, torch.float32, True),
                                                      (torch.bfloat16, torch.bfloat16, True),
                                                      (torch.float32, torch.bfloat16, False),
                                                      (torch.bfloat16, torch.float32, True)])
def test_step_multi_tensor_ragged(sv, g_dtype, x_dtype, momentum, two_kernels):
    # 60 tensors of ragged sizes, every worker's gradient / momentum of every tensor an allocation of its own;
    # every fifth tensor sits at an odd element offset (no vector alignment: the one-element-per-lane path).
    # ONE launch per step -- or, with a workspace for the packed signs, the two-kernel form, whose workspace must
    # then hold exactly what every worker transmitted.  The oracle runs Algorithm 1 tensor by tensor.
    M, T, steps = 7, 60, 3
    beta = 0.9 if momentum else 0.0
    lr, wd = (1e-4, 0.0) if x_dtype == torch.float32 else (1e-5, 0.0)
    rng = np.random.default_rng(60)
    sizes = _ragged_sizes(rng, T)
    _log(f"multi-tensor step g={g_dtype} x={x_dtype} momentum={momentum}: {T} tensors, {sum(sizes)} coordinates")

    def alloc(n, dtype, t, fill):
        off = 1 if t % 5 == 4 else 0                          # misaligned view for every fifth tensor
        buf = torch.full((n + 9,), fill, dtype=dtype, device=DEV)
        return buf, buf[off:off + n]

    xbufs, params = zip(*[alloc(n, x_dtype, t, 7.0) for t, n in enumerate(sizes)])
    for t, p in enumerate(params):
        p.copy_(wl.gaussian((sizes[t],), 0.02, seed=100 + t, device=DEV))
    gbufs, grads, vbufs, moms = [], [], [], []
    for m in range(M):
        b, g = zip(*[alloc(n, g_dtype, t, 3.0) for t, n in enumerate(sizes)])
        gbufs.append(b), grads.append(list(g))
        if momentum:
            b, v = zip(*[alloc(n, torch.float32, t, 0.0) for t, n in enumerate(sizes)])
            vbufs.append(b), moms.append(list(v))
    plan = sv.MultiTensorPlan(list(params), grads, moms if momentum else None)
    assert plan.numel == sum(sizes) and plan.T == T and plan.M == M
    ws = None
    units = [(n + 4095) // 4096 for n in sizes]
    first_unit = np.concatenate([[0], np.cumsum(units)])
    if two_kernels:
        ws = sv.multi_workspace(plan)
        assert ws.numel() == M * 64 * int(first_unit[-1])
        ws.fill_(-1)                                           # stale contents must not matter
    x_ref = [wl.to_numpy(p.contiguous()).copy() for p in params]
    v_ref = [np.zeros((M, n), np.float32) for n in sizes] if momentum else [None] * T
    mus = [wl.shared_mean(n, seed=500 + t, device=DEV) for t, n in enumerate(sizes)]
    for step in range(steps):
        for t, n in enumerate(sizes):
            gt = wl.worker_gradients(mus[t], M, step, base_seed=9000 + 31 * t, dtype=g_dtype)
            for m in range(M):
                grads[m][t].copy_(gt[m])
        sv.signum_step_multi(plan, beta, lr, wd, workspace=ws)
        torch.cuda.synchronize()
        ws_h = None if ws is None else wl.to_numpy(ws).view(np.uint64).reshape(M, -1)
        for t, n in enumerate(sizes):
            g_h = np.stack([wl.to_numpy(grads[m][t].contiguous()) for m in range(M)])
            _, signs_ref = ora.signum_step(g_h, v_ref[t], beta, x_ref[t], lr, wd, want_signs=True)
            assert np.array_equal(wl.to_numpy(params[t].contiguous()), x_ref[t]), f"weights of tensor {t} (n={n}), step {step}"
            if ws_h is not None:
                w0 = 64 * int(first_unit[t])
                assert np.array_equal(ws_h[:, w0:w0 + signs_ref.shape[1]], signs_ref), f"packed signs of tensor {t} (n={n})"
            if momentum:
                v_gpu = np.stack([wl.to_numpy(moms[m][t].contiguous()) for m in range(M)])
                assert np.array_equal(v_gpu, v_ref[t]), f"momentum of tensor {t} (n={n}), step {step}"
    # nothing outside the tensors was touched: guard elements keep their fill
    for t, n in enumerate(sizes):
        off = 1 if t % 5 == 4 else 0
        assert (xbufs[t][:off] == 7.0).all() and (xbufs[t][off + n:] == 7.0).all(), f"wrote outside weights {t}"
        for m in range(M):
            assert (gbufs[m][t][off + n:] == 3.0).all()
            if momentum:
                assert (vbufs[m][t][:off] == 0.0).all() and (vbufs[m][t][off + n:] == 0.0).all(), f"outside momentum {t}"


def test_step_multi_equals_flat_step_on_one_large_tensor(sv):
    # a single tensor: the multi-tensor launch must equal the flat fused step bit for bit, ragged end included
    M, d = 15, 300_007
    mu = wl.shared_mean(d, seed=1, device=DEV)
    g = wl.worker_gradients(mu, M, 0, base_seed=77)
    x_flat = wl.gaussian((d,), 0.02, seed=2, device=DEV)
    x_multi = x_flat.clone()
    v_flat = torch.zeros((M, d), device=DEV)
    v_rows = [torch.zeros((d,), device=DEV) for _ in range(M)]
    plan = sv.MultiTensorPlan([x_multi], [[g[m].clone()] for m in range(M)], [[v_rows[m]] for m in range(M)])
    x_ws = x_flat.clone()
    v_ws = [torch.zeros((d,), device=DEV) for _ in range(M)]
    plan_ws = sv.MultiTensorPlan([x_ws], [[g[m].clone()] for m in range(M)], [[v_ws[m]] for m in range(M)])
    ws = sv.multi_workspace(plan_ws)
    for _ in range(3):
        sv.signum_step(g, v_flat, 0.9, x_flat, 1e-4)
        sv.signum_step_multi(plan, 0.9, 1e-4)
        sv.signum_step_multi(plan_ws, 0.9, 1e-4, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(x_flat, x_multi) and torch.equal(x_flat, x_ws)
    assert all(torch.equal(v_flat[m], v_rows[m]) and torch.equal(v_flat[m], v_ws[m]) for m in range(M))
    with pytest.raises(sv.SignvoteError):
        sv.signum_step_multi(plan_ws, 0.9, 1e-4, workspace=ws[:-1])         # one word short


@pytest.mark.parametrize("M", [17, 70, 300])
def test_step_multi_worker_counts_beyond_15(sv, M):
    # the vote of the two-kernel multi-tensor form keeps 4 / 6 / 8 / 10 bit planes for M <= 15 / 63 / 255 / 1023:
    # both multi-tensor forms against the oracle on a few ragged tensors for the larger counters
    sizes = [1, 65, 4097, 9000, 256, 70_000]
    beta, lr = 0.9, 1e-4
    mus = [wl.shared_mean(n, seed=300 + t, device=DEV) for t, n in enumerate(sizes)]
    grads = [[torch.empty(n, device=DEV) for n in sizes] for _ in range(M)]
    state = {}
    for form in ("one", "two"):
        params = [wl.gaussian((n,), 0.02, seed=400 + t, device=DEV) for t, n in enumerate(sizes)]
        moms = [[torch.zeros(n, device=DEV) for n in sizes] for _ in range(M)]
        plan = sv.MultiTensorPlan(params, grads, moms)
        state[form] = (params, moms, plan, sv.multi_workspace(plan) if form == "two" else None)
    x_ref = [wl.to_numpy(p).copy() for p in state["one"][0]]
    v_ref = [np.zeros((M, n), np.float32) for n in sizes]
    for step in range(2):
        for t, n in enumerate(sizes):
            gt = wl.worker_gradients(mus[t], M, step, base_seed=7000 + 13 * t)
            for m in range(M):
                grads[m][t].copy_(gt[m])
        for form in ("one", "two"):
            _, _, plan, ws = state[form]
            sv.signum_step_multi(plan, beta, lr, workspace=ws)
        torch.cuda.synchronize()
        for t, n in enumerate(sizes):
            g_h = np.stack([wl.to_numpy(grads[m][t]) for m in range(M)])
            ora.signum_step(g_h, v_ref[t], beta, x_ref[t], lr)
            for form in ("one", "two"):
                params, moms, _, _ = state[form]
                assert np.array_equal(wl.to_numpy(params[t]), x_ref[t]), f"{form}-kernel form, weights of tensor {t}, step {step}"
                v_gpu = np.stack([wl.to_numpy(moms[m][t]) for m in range(M)])
                assert np.array_equal(v_gpu, v_ref[t]), f"{form}-kernel form, momentum of tensor {t}, step {step}"


def test_multi_plan_rejects_bad_tensor_lists(sv):
    x = [torch.zeros(10, device=DEV), torch.zeros(20, device=DEV)]
    g = [[torch.zeros(10, device=DEV), torch.zeros(20, device=DEV)] for _ in range(3)]
    with pytest.raises(ValueError):
        sv.MultiTensorPlan(x, [row[:1] for row in g])                       # a worker misses a tensor
    with pytest.raises(ValueError):
        sv.MultiTensorPlan(x, [[torch.zeros(10, device=DEV), torch.zeros(21, device=DEV)]] * 3)   # size mismatch
    with pytest.raises(ValueError):
        sv.MultiTensorPlan(x, g, [[t.to(torch.bfloat16) for t in row] for row in g])                # momentum must be fp32
    with pytest.raises(ValueError):
        sv.MultiTensorPlan([torch.zeros(4, 4, device=DEV).T, x[1]], g)                             # not contiguous
    plan = sv.MultiTensorPlan(x, g)                                                                   # signSGD plan
    with pytest.raises(sv.SignvoteError) as e:
        sv.signum_step_multi(plan, 0.9, 1e-3)                                                        # momentum without v
    assert e.value.status == -5


def test_argument_errors_leave_buffers_untouched(sv):
    lib = sv.load_library()
    d, M = 1000, 3
    g = wl.gaussian((M, d), 1.0, seed=1, device=DEV)
    x = wl.gaussian((d,), 0.02, seed=2, device=DEV)
    x0 = x.clone()
    signs = torch.full((M, sv.words_for(d)), 7, dtype=torch.int64, device=DEV)
    with pytest.raises(sv.SignvoteError) as e:
        sv.signum_step(g, None, 0.9, x, 1e-3)             # momentum asked without v
    assert e.value.status == -5
    assert lib.ssv_sign_pack(g.data_ptr(), 0, 0, d, d, signs.data_ptr(), signs.stride(0), None) == -2
    assert lib.ssv_sign_pack(g.data_ptr(), 0, M, d, d - 1, signs.data_ptr(), signs.stride(0), None) == -2
    assert lib.ssv_sign_pack(g.data_ptr(), 5, M, d, d, signs.data_ptr(), signs.stride(0), None) == -4
    assert lib.ssv_sign_pack(g.data_ptr() + 2, 0, M, d, d, signs.data_ptr(), signs.stride(0), None) == -3
    assert lib.ssv_majority_vote(signs.data_ptr(), 1024, d, signs.stride(0), signs.data_ptr(), None) == -2
    assert lib.ssv_apply_sign_update(x.data_ptr(), 0, d, signs.data_ptr(), float("nan"), 0.0, None) == -5
    torch.cuda.synchronize()
    assert torch.equal(x, x0) and (signs == 7).all()


def test_step_randomised_shapes(sv):
    # seeded sweep over worker counts, lengths, paddings, dtypes and options
    rng = np.random.default_rng(2024)
    dtypes = [torch.float32, torch.bfloat16]
    for case in range(48):
        M = int(rng.integers(1, 70))
        d = int(rng.integers(1, 6000))
        pad = int(rng.choice([0, 0, 1, 3, 4, 8, 29]))
        g_dt, x_dt = dtypes[int(rng.integers(2))], dtypes[int(rng.integers(2))]
        momentum = bool(rng.integers(4) > 0)
        beta = float(rng.choice([0.0, 0.5, 0.9, 0.99])) if momentum else 0.0
        wd = float(rng.choice([0.0, 0.0, 0.01]))
        flip = [int(b) for b in rng.integers(0, 2, size=M)] if rng.integers(3) == 0 else None
        x_off = int(rng.choice([0, 0, 1, 4]))
        _log(f"random case {case}: M={M} d={d} pad={pad} g={g_dt} x={x_dt} beta={beta} wd={wd} "
             f"flip={'yes' if flip else 'no'} x_off={x_off} momentum={momentum}")
        assert _step_case(sv, M, d, g_dt, x_dt, beta, wd, steps=2, pad=pad, flip=flip, momentum=momentum,
                          x_off=x_off) == 0


def test_vote_randomised_shapes(sv):
    rng = np.random.default_rng(77)
    for case in range(40):
        M = int(rng.integers(1, 300))
        d = int(rng.integers(1, 40000))
        extra = int(rng.integers(0, 4))
        W = sv.words_for(d)
        _log(f"random vote case {case}: M={M} d={d} stride={W + extra}")
        rows = wl.random_words((M, W + extra), seed=1000 + case, device=DEV)[:, :W]
        x = wl.gaussian((d + 3,), 0.02, seed=case, device=DEV)[int(rng.integers(0, 2)):][:d]
        x_h = wl.to_numpy(x.contiguous()).copy()
        vote_buf = torch.full((W + 2,), -1, dtype=torch.int64, device=DEV)
        sv.majority_vote(rows, d, vote_buf[:W])
        vote2 = torch.full((W,), -1, dtype=torch.int64, device=DEV)
        sv.vote_apply(rows, d, x, 1e-3, 0.0, vote_out=vote2)
        torch.cuda.synchronize()
        ref = ora.vote_apply(_np_rows(rows), d, x_h, 1e-3, 0.0)
        assert np.array_equal(wl.to_numpy(vote_buf[:W]), ref) and np.array_equal(wl.to_numpy(vote2), ref)
        assert (vote_buf[W:] == -1).all()
        assert np.array_equal(wl.to_numpy(x.contiguous()), x_h)
