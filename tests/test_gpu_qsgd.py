"""GPU parity of the ternary QSGD compressors (include/signvote_qsgd.h) against the CPU oracle, through the C ABI.
Bars: the packed codes and the max norm are bit-exact; the Euclidean norm is within 1e-6 relative (both sides sum
exact squares in double precision, in different orders, and round once to fp32: they are expected to be equal, and
the test reports when they are not); averages and weights are bit-identical to the oracle's fp32 evaluation, which
fixes the same operation order."""
import math

import numpy as np
import pytest
import torch

import oracle as ora
import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
KINDS = [ora.QSGD_L2, ora.QSGD_MAX]


@pytest.fixture(scope="module")
def sv():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_1810_05291_amd as sv_
    sv_.load_library()
    assert (sv_.SSV_QSGD_L2, sv_.SSV_QSGD_MAX) == (ora.QSGD_L2, ora.QSGD_MAX)
    return sv_


def _log(*a):
    print(*a, flush=True)


def _host(t):
    return np.ascontiguousarray(wl.to_numpy(t.contiguous()))


def _strided(rows, cols, stride, dtype, fill):
    buf = torch.full((rows, stride), fill, dtype=dtype, device=DEV)
    return buf, buf[:, :cols]


def _uniform(shape, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    return torch.rand(shape, device=DEV, generator=g)


RAGGED_D = [1, 3, 63, 64, 65, 255, 256, 257, 1000, 4095, 4096, 4097, 65_536, 100_003, 1_048_577]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kind", KINDS)
def test_norms_ragged(sv, kind, dtype):
    unequal = 0
    for d in RAGGED_D:
        for M, pad in ((1, 0), (3, 0), (5, 1), (4, 12)):
            _log(f"qsgd_norms kind={kind} dtype={dtype} d={d} M={M} pad={pad}")
            buf, g = _strided(M, d, d + pad, dtype, 1e30)              # huge pads: must not be read
            g.copy_(wl.gaussian((M, d), 1e-2, seed=d + M, device=DEV))
            norms = sv.qsgd_norms(g, kind)
            torch.cuda.synchronize()
            ref = ora.qsgd_norms(_host(g), kind)
            got = _host(norms)
            if kind == ora.QSGD_MAX:
                assert np.array_equal(got, ref)
            else:
                assert (np.abs(got.astype(np.float64) - ref) <= 1e-6 * ref).all()
                unequal += int((got != ref).sum())
    _log(f"qsgd_norms kind={kind} dtype={dtype}: norms that differ from the oracle's in the last place: {unequal}")
    assert unequal == 0


def test_norms_special_values_and_workspace_reuse(sv):
    M, d = 4, 5000
    g = wl.gaussian((M, d), 1.0, seed=3, device=DEV)
    g[1, 17] = float("nan")
    g[2, :] = 0.0
    g[3, 4000] = -1e30
    ws = sv.qsgd_workspace(M, DEV)
    ws.fill_(float("nan"))                                      # stale contents must not matter
    for kind in KINDS:
        out = torch.full((M,), -1.0, device=DEV)
        sv.qsgd_norms(g, kind, norms=out, workspace=ws)
        torch.cuda.synchronize()
        got, ref = _host(out), ora.qsgd_norms(_host(g), kind)
        assert np.array_equal(np.isnan(got), np.isnan(ref))
        assert np.array_equal(got[~np.isnan(ref)], ref[~np.isnan(ref)])
        assert got[2] == 0.0
    assert np.isnan(ora.qsgd_norms(_host(g), ora.QSGD_L2)[1]) and not np.isnan(ora.qsgd_norms(_host(g), ora.QSGD_MAX)[1])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("kind", KINDS)
def test_quantize_ragged_bit_exact(sv, kind, dtype):
    for d in RAGGED_D:
        for M, gpad, upad, wpad in ((1, 0, 0, 0), (3, 0, 0, 1), (5, 1, 3, 2), (4, 12, 8, 0)):
            _log(f"qsgd_quantize kind={kind} dtype={dtype} d={d} M={M} pads={gpad},{upad},{wpad}")
            _, g = _strided(M, d, d + gpad, dtype, 7.0)
            g.copy_(wl.gaussian((M, d), 1e-2, seed=2 * d + M, device=DEV))
            g[:, ::9] = 0.0
            _, u = _strided(M, d, d + upad, torch.float32, 0.0)
            u.copy_(_uniform((M, d), seed=d))
            g_h, u_h = _host(g), _host(u)
            norms_h = ora.qsgd_norms(g_h, kind)                       # both sides quantise against the same scale
            W = sv.words_for(d)
            nzbuf, nz = _strided(M, W, W + wpad, torch.int64, -1)
            sgbuf, sg = _strided(M, W, W + wpad, torch.int64, -1)
            sv.qsgd_quantize(g, u, torch.from_numpy(norms_h).to(DEV), nz, sg)
            torch.cuda.synchronize()
            nz_ref, sg_ref = ora.qsgd_quantize(g_h, u_h, norms_h)
            assert np.array_equal(_host(nz), nz_ref) and np.array_equal(_host(sg), sg_ref)
            assert (nzbuf[:, W:] == -1).all() and (sgbuf[:, W:] == -1).all(), "wrote past the row"


def test_quantize_special_values_and_extreme_draws(sv):
    M, d = 3, 1024
    g = wl.gaussian((M, d), 1.0, seed=5, device=DEV)
    g[0, :100] = float("nan")
    g[0, 100:200] = float("inf")
    g[0, 200:300] = float("-inf")
    g[1, ::2] = 0.0
    g[1, 1::4] = -0.0
    g[2, :64] = 1e-45                                              # denormals are numbers: kept with probability |g| / norm
    u = _uniform((M, d), seed=6)
    u[2, :32] = 0.0
    u[:, 500:600] = 0.0                                            # u = 0 keeps every non-zero number
    for norms_h in (np.array([np.inf, 2.5, 1e-40], np.float32), np.array([3.0, 0.0, 4.0], np.float32)):
        nz, sg = sv.qsgd_quantize(g, u, torch.from_numpy(norms_h).to(DEV))
        torch.cuda.synchronize()
        nz_ref, sg_ref = ora.qsgd_quantize(_host(g), _host(u), norms_h)
        assert np.array_equal(_host(nz), nz_ref) and np.array_equal(_host(sg), sg_ref)
    # max QSGD leaves a sign vector unchanged (Appendix B)
    s = torch.where(_uniform((1, 4096), seed=7) < 0.5, -1.0, 1.0)
    norms = sv.qsgd_norms(s, sv.SSV_QSGD_MAX)
    nz, sg = sv.qsgd_quantize(s, _uniform((1, 4096), seed=8), norms)
    torch.cuda.synchronize()
    assert (_host(nz) == np.uint64(0xFFFFFFFFFFFFFFFF)).all()
    assert np.array_equal(_host(sg), ora.sign_pack(_host(s)))


@pytest.mark.parametrize("x_dtype", [torch.float32, torch.bfloat16])
def test_aggregate_apply_ragged_bit_exact(sv, x_dtype):
    rng = np.random.default_rng(8)
    for d in RAGGED_D:
        for M, wpad, off in ((1, 0, 0), (3, 1, 0), (15, 0, 1), (40, 2, 0)):
            _log(f"qsgd_aggregate_apply x={x_dtype} d={d} M={M} wpad={wpad} off={off}")
            W = sv.words_for(d)
            nz = wl.random_words((M, W + wpad), seed=d + M, device=DEV)[:, :W]
            sg_full = wl.random_words((M, W + wpad), seed=d + M + 1, device=DEV)
            sg = (sg_full & wl.random_words((M, W + wpad), seed=0, device=DEV))[:, :W]   # any bits: consumers read sign only where nonzero
            norms_h = (rng.random(M) * 2 + 0.01).astype(np.float32)
            norms = torch.from_numpy(norms_h).to(DEV)
            xbuf = wl.gaussian((d + 8,), 0.02, seed=9, device=DEV).to(x_dtype)
            x = xbuf[off:off + d]
            x_ref = _host(x).copy()
            abuf = torch.full((d + 8,), -5.0, device=DEV)
            avg = abuf[off:off + d] if off == 0 else abuf[4:4 + d]
            lr = 0.05
            sv.qsgd_aggregate_apply(nz, sg, norms, d, avg_out=avg, x=x, lr=lr)
            x2 = xbuf.clone()[off:off + d]                                # second form: update only, from the updated x
            torch.cuda.synchronize()
            avg_ref = ora.qsgd_aggregate_apply(_host(nz), _host(sg), norms_h, d, x_ref, lr)
            assert np.array_equal(_host(avg), avg_ref), "average differs"
            assert np.array_equal(_host(x), x_ref), "weights differ"
            # float64 evaluation: within fp32 rounding of the exact average
            q = np.stack([ora.qsgd_unpack(_host(nz)[m], _host(sg)[m], d) for m in range(M)])
            exact = (q.astype(np.float64) * norms_h.astype(np.float64)[:, None]).sum(axis=0) / M
            scale = np.abs(q.astype(np.float64) * norms_h[:, None]).sum(axis=0) / M
            assert (np.abs(_host(avg) - exact) <= 1e-6 * scale + 1e-30).all()
            # guards untouched
            ref_buf = wl.gaussian((d + 8,), 0.02, seed=9, device=DEV).to(x_dtype)
            assert torch.equal(xbuf[:off], ref_buf[:off]) and torch.equal(xbuf[off + d:], ref_buf[off + d:])
            a0 = 0 if off == 0 else 4
            assert (abuf[:a0] == -5.0).all() and (abuf[a0 + d:] == -5.0).all()
            # update only / average only forms agree with the combined one
            x_only = ref_buf[off:off + d].clone()
            sv.qsgd_aggregate_apply(nz, sg, norms, d, x=x_only, lr=lr)
            a_only = torch.empty((d,), device=DEV)
            sv.qsgd_aggregate_apply(nz, sg, norms, d, avg_out=a_only)
            torch.cuda.synchronize()
            assert torch.equal(x_only, x) and torch.equal(a_only, avg)
            del x2


@pytest.mark.timeout(600)
@pytest.mark.parametrize("M", [3, 15])
def test_qsgd_full_pipeline_resnet50_size(sv, M):
    # the whole 1-way scheme at the resnet50 size, each side from its own norms: norm, quantise, average + update.
    # M = 3 is the worker count of the paper's QSGD figure, M = 15 the headline workload's.
    d = wl.RESNET50_D
    stride = ((d + 31) // 32) * 32
    mu = wl.shared_mean(d, seed=1, device=DEV)
    g = wl.worker_gradients(mu, M, 0, base_seed=6000, row_stride=stride)
    u = torch.empty((M, stride), device=DEV)[:, :d]
    for m in range(M):
        u[m] = _uniform((d,), seed=700 + m)
    g_h, u_h = _host(g), _host(u)
    x0 = wl.gaussian((d,), 0.02, seed=2, device=DEV)
    W = sv.words_for(d)
    for kind, name in ((ora.QSGD_L2, "L2"), (ora.QSGD_MAX, "max")):
        norms = sv.qsgd_norms(g, kind)
        nz, sg = sv.qsgd_quantize(g, u, norms)
        x = x0.clone()
        avg = torch.empty((d,), device=DEV)
        sv.qsgd_aggregate_apply(nz, sg, norms, d, avg_out=avg, x=x, lr=0.1)
        torch.cuda.synchronize()
        norms_ref = ora.qsgd_norms(g_h, kind)
        got_norms = _host(norms)
        assert (np.abs(got_norms.astype(np.float64) - norms_ref) <= 1e-6 * norms_ref).all()
        assert np.array_equal(got_norms, norms_ref), "a norm differs in the last place: codes may then differ"
        nz_ref, sg_ref = ora.qsgd_quantize(g_h, u_h, norms_ref)
        assert np.array_equal(_host(nz), nz_ref) and np.array_equal(_host(sg), sg_ref)
        x_ref = _host(x0).copy()
        avg_ref = ora.qsgd_aggregate_apply(nz_ref, sg_ref, norms_ref, d, x_ref, 0.1)
        assert np.array_equal(_host(avg), avg_ref) and np.array_equal(_host(x), x_ref)
        # Appendix B's accounting on this input
        nnz = np.array([int(np.unpackbits(nz_ref[m].view(np.uint8)).sum()) for m in range(M)])
        l1_over_l2 = np.abs(g_h.astype(np.float64)).sum(axis=1) / norms_ref
        sparse_bits = nnz * (1 + math.ceil(math.log2(d)))
        _log(f"QSGD {name}, d={d}, M={M}: kept per worker {nnz.mean():.0f} of {d} ({nnz.mean() / d:.5f}); "
             f"as (index, sign) pairs {sparse_bits.mean() / 8e6:.2f} MB per worker vs {d / 8e6:.2f} MB for a sign vector "
             f"and {2 * d / 8e6:.2f} MB for the two bit planes")
        if kind == ora.QSGD_L2:
            assert (nnz <= 1.02 * math.sqrt(d)).all()                          # E[#] = |g|_1 / |g|_2 <= sqrt(d)
            assert (np.abs(nnz - l1_over_l2) <= 6 * np.sqrt(l1_over_l2)).all()
        else:
            expect = np.abs(g_h.astype(np.float64)).sum(axis=1) / norms_ref
            assert (np.abs(nnz - expect) <= 6 * np.sqrt(expect)).all()


def test_one_way_qsgd_sgd_follows_the_oracle_on_the_toy_quadratic(sv):
    # f(x) = |x|^2 / 2 in 1000 dimensions, gradient noise N(0, 1), M = 3: SGD on the averaged decoded gradients.  Each
    # side runs its own closed loop from its own weights; the noise and the uniform draws are the shared inputs.
    M, d, lr, steps = 3, 1000, 0.05, 150
    for kind in KINDS:
        x = wl.gaussian((d,), 1.0, seed=50, device=DEV)
        x_ref = _host(x).copy()
        start = float((x_ref.astype(np.float64) ** 2).sum())
        ws = sv.qsgd_workspace(M, DEV)
        for k in range(steps):
            noise = wl.gaussian((M, d), 1.0, seed=51 + k, device=DEV)
            u = _uniform((M, d), seed=9000 + k)
            g = (x[None, :] + noise).contiguous()
            g_h = (x_ref[None, :] + _host(noise)).astype(np.float32)
            norms = sv.qsgd_norms(g, kind, workspace=ws)
            nz, sg = sv.qsgd_quantize(g, u, norms)
            sv.qsgd_aggregate_apply(nz, sg, norms, d, x=x, lr=lr)
            torch.cuda.synchronize()
            norms_ref = ora.qsgd_norms(g_h, kind)
            nz_ref, sg_ref = ora.qsgd_quantize(g_h, _host(u), norms_ref)
            ora.qsgd_aggregate_apply(nz_ref, sg_ref, norms_ref, d, x_ref, lr)
            assert np.array_equal(_host(x), x_ref), f"trajectory left the oracle's at step {k} (kind {kind})"
        end = float((x_ref.astype(np.float64) ** 2).sum())
        _log(f"1-way QSGD kind={kind}: |x|^2 {start:.1f} -> {end:.2f} in {steps} steps")
        assert end < 0.3 * start
