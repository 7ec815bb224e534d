"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the public
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "signvote.h"), os.path.join(ROOT, "include", "signvote_bench.h"),
           os.path.join(ROOT, "include", "signvote_qsgd.h")]


@pytest.fixture(scope="module")
def lib():
    import paper_1810_05291_amd as sv
    if not os.path.exists(sv.library_path()):
        from paper_1810_05291_amd import build
        build.build()
    return sv.load_library()


def _declared_symbols():
    names = set()
    for header in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(ssv_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(lib):
    names = _declared_symbols()
    assert {"ssv_sign_pack", "ssv_signum_momentum_pack", "ssv_majority_vote", "ssv_apply_sign_update",
            "ssv_vote_apply", "ssv_signum_step", "ssv_status_string", "ssv_version", "ssv_bench_copy",
            "ssv_multi_plan_bytes", "ssv_multi_plan_fill", "ssv_signum_step_multi",
            "ssv_multi_workspace_bytes", "ssv_signum_step_multi_ws", "ssv_qsgd_norms_static",
            "ssv_qsgd_workspace_bytes", "ssv_qsgd_norms", "ssv_qsgd_quantize", "ssv_qsgd_aggregate_apply"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in signvote.h but not exported"


def test_version_and_status_strings(lib):
    assert lib.ssv_version() >= 1000
    seen = set()
    for code in range(0, -7, -1):
        s = lib.ssv_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert b"unknown" in lib.ssv_status_string(-99)


def test_argument_validation_needs_no_device(lib):
    # fake but well-aligned addresses: validation must fail before any dereference or launch
    P = 0x1000
    W = 16
    assert lib.ssv_sign_pack(None, 0, 3, 1000, 1000, P, W, None) == -1
    assert lib.ssv_sign_pack(P, 0, 3, 1000, 1000, None, W, None) == -1
    assert lib.ssv_sign_pack(P, 0, 0, 1000, 1000, P, W, None) == -2
    assert lib.ssv_sign_pack(P, 0, 1024, 1000, 1000, P, W, None) == -2
    assert lib.ssv_sign_pack(P, 0, 3, 0, 1000, P, W, None) == -2
    assert lib.ssv_sign_pack(P, 0, 3, (1 << 40) + 1, 1 << 41, P, 1 << 40, None) == -2
    assert lib.ssv_sign_pack(P, 0, 3, 1000, 999, P, W, None) == -2
    assert lib.ssv_sign_pack(P, 0, 3, 1000, 1000, P, 15, None) == -2
    assert lib.ssv_sign_pack(P, 2, 3, 1000, 1000, P, W, None) == -4
    assert lib.ssv_sign_pack(P + 2, 0, 3, 1000, 1000, P, W, None) == -3
    assert lib.ssv_sign_pack(P, 0, 3, 1000, 1000, P + 4, W, None) == -3
    assert lib.ssv_signum_momentum_pack(P, 0, None, 3, 1000, 1000, 1000, 0.9, P, W, None) == -1
    assert lib.ssv_signum_momentum_pack(P, 0, P, 3, 1000, 1000, 1000, 1.0, P, W, None) == -5
    assert lib.ssv_signum_momentum_pack(P, 0, P, 3, 1000, 1000, 1000, -0.1, P, W, None) == -5
    assert lib.ssv_signum_momentum_pack(P, 0, P, 3, 1000, 1000, 1000, float("nan"), P, W, None) == -5
    assert lib.ssv_signum_momentum_pack(P, 0, P, 3, 1000, 1000, 10, 0.9, P, W, None) == -2
    assert lib.ssv_majority_vote(None, 3, 1000, W, P, None) == -1
    assert lib.ssv_majority_vote(P, 3, 1000, W, None, None) == -1
    assert lib.ssv_majority_vote(P, 3, 1000, 15, P, None) == -2
    assert lib.ssv_majority_vote(P + 4, 3, 1000, W, P, None) == -3
    assert lib.ssv_apply_sign_update(None, 0, 1000, P, 1e-3, 0.0, None) == -1
    assert lib.ssv_apply_sign_update(P, 0, 1000, P, float("inf"), 0.0, None) == -5
    assert lib.ssv_apply_sign_update(P, 0, 1000, P, 1e-3, float("nan"), None) == -5
    assert lib.ssv_apply_sign_update(P, 7, 1000, P, 1e-3, 0.0, None) == -4
    assert lib.ssv_apply_sign_update(P + 1, 1, 1000, P, 1e-3, 0.0, None) == -3
    assert lib.ssv_vote_apply(P, 3, 1000, W, None, 0, 1e-3, 0.0, None, None) == -1
    assert lib.ssv_vote_apply(P, 3, 1000, W, P, 3, 1e-3, 0.0, None, None) == -4
    assert lib.ssv_signum_step(P, 0, None, 3, 1000, 1000, 0, 0.9, P, 0, 1e-3, 0.0, None, None, 0, None, None) == -5
    assert lib.ssv_signum_step(P, 0, P, 3, 1000, 1000, 1000, 0.9, None, 0, 1e-3, 0.0, None, None, 0, None, None) == -1
    assert lib.ssv_signum_step(P, 0, P, 3, 1000, 1000, 1000, 0.9, P, 0, 1e-3, 0.0, None, P, 3, None, None) == -2
    assert lib.ssv_bench_copy(None, P, 1024, None) == -1
    assert lib.ssv_bench_copy(P, P + 4096, 1000, None) == -2
    assert lib.ssv_bench_copy(P + 8, P + 4096, 1024, None) == -3


def test_multi_tensor_plan_is_built_on_the_host(lib):
    # the plan is sized and filled without touching a device: fake (aligned) device addresses suffice
    import numpy as np
    lib.ssv_multi_plan_bytes.restype = ctypes.c_size_t
    T, M = 5, 3
    n_list = [1, 63, 4096, 4097, 10_000]                    # 1 + 1 + 1 + 2 + 3 = 8 units of 4096 coordinates
    n = (ctypes.c_int64 * T)(*n_list)
    nbytes = lib.ssv_multi_plan_bytes(T, M, n)
    assert nbytes > 0 and nbytes % 8 == 0
    assert lib.ssv_multi_plan_bytes(0, M, n) == 0 and lib.ssv_multi_plan_bytes(T, 0, n) == 0
    assert lib.ssv_multi_plan_bytes(T, 1024, n) == 0 and lib.ssv_multi_plan_bytes(T, M, None) == 0
    bad = (ctypes.c_int64 * T)(1, 0, 5, 5, 5)
    assert lib.ssv_multi_plan_bytes(T, M, bad) == 0
    huge = (ctypes.c_int64 * 2)(1 << 40, 1)                  # sum beyond the coordinate limit
    assert lib.ssv_multi_plan_bytes(2, M, huge) == 0
    # more tensors, more workers or more units need more bytes
    assert lib.ssv_multi_plan_bytes(T, M + 1, n) > nbytes
    n2 = (ctypes.c_int64 * T)(1, 63, 4096, 4097, 10_000 + 400_000)
    assert lib.ssv_multi_plan_bytes(T, M, n2) > nbytes

    xs = (ctypes.c_void_p * T)(*[0x10000 * (t + 1) for t in range(T)])
    gs = (ctypes.c_void_p * (T * M))(*[0x1000000 + 0x10000 * k for k in range(T * M)])
    vs = (ctypes.c_void_p * (T * M))(*[0x9000000 + 0x10000 * k for k in range(T * M)])
    buf = np.zeros(nbytes // 8 + 1, np.int64)
    host = buf.ctypes.data
    fill = lib.ssv_multi_plan_fill
    assert fill(host, nbytes, T, M, n, xs, 0, gs, 0, vs) == 0
    words = buf.view(np.uint64)
    assert bytes(words[:1].tobytes()) == b"SSVPLAN1"
    assert int(words[1]) == nbytes and [int(w) for w in words[2:6]] == [T, M, 8, sum(n_list)]
    assert buf[nbytes // 8] == 0                                              # nothing written past the stated size
    # argument errors
    assert fill(None, nbytes, T, M, n, xs, 0, gs, 0, vs) == -1
    assert fill(host, nbytes, T, M, n, None, 0, gs, 0, vs) == -1
    assert fill(host, nbytes, T, M, n, xs, 0, None, 0, vs) == -1
    assert fill(host, nbytes - 8, T, M, n, xs, 0, gs, 0, vs) == -2
    assert fill(host, nbytes, T, M, bad, xs, 0, gs, 0, vs) == -2
    assert fill(host, nbytes, T, M, n, xs, 2, gs, 0, vs) == -4
    assert fill(host, nbytes, T, M, n, xs, 0, gs, 7, vs) == -4
    assert fill(host + 4, nbytes, T, M, n, xs, 0, gs, 0, vs) == -3
    gs_bad = (ctypes.c_void_p * (T * M))(*[0x1000000 + 0x10000 * k + (2 if k == 7 else 0) for k in range(T * M)])
    assert fill(host, nbytes, T, M, n, xs, 0, gs_bad, 0, vs) == -3           # fp32 gradient at an odd half-word
    assert fill(host, nbytes, T, M, n, xs, 0, gs_bad, 1, vs) == 0            # fine for bf16
    gs_null = (ctypes.c_void_p * (T * M))(*[0x1000000 + 0x10000 * k if k != 4 else 0 for k in range(T * M)])
    assert fill(host, nbytes, T, M, n, xs, 0, gs_null, 0, vs) == -1
    # the step validates its arguments before any launch
    step = lib.ssv_signum_step_multi
    step.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
    assert fill(host, nbytes, T, M, n, xs, 0, gs, 0, vs) == 0
    assert step(None, 0x1000, 0.9, 1e-3, 0.0, None) == -1
    assert step(host, None, 0.9, 1e-3, 0.0, None) == -1
    assert step(host, 0x1004, 0.9, 1e-3, 0.0, None) == -3
    assert step(host, 0x1000, 1.0, 1e-3, 0.0, None) == -5
    assert step(host, 0x1000, 0.9, float("inf"), 0.0, None) == -5
    junk = np.zeros(64, np.int64)
    assert step(junk.ctypes.data, 0x1000, 0.9, 1e-3, 0.0, None) == -2         # not a plan
    # the two-kernel form: its workspace holds 64 words per unit and worker
    wsb = lib.ssv_multi_workspace_bytes
    wsb.argtypes, wsb.restype = [ctypes.c_void_p], ctypes.c_size_t
    assert wsb(host) == M * 8 * 64 * 8 and wsb(None) == 0 and wsb(junk.ctypes.data) == 0
    step_ws = lib.ssv_signum_step_multi_ws
    step_ws.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_float,
                        ctypes.c_float, ctypes.c_void_p]
    need = wsb(host)
    assert step_ws(host, 0x1000, None, need, 0.9, 1e-3, 0.0, None) == -1
    assert step_ws(host, 0x1000, 0x2008, need, 0.9, 1e-3, 0.0, None) == -3
    assert step_ws(host, 0x1000, 0x2000, need - 1, 0.9, 1e-3, 0.0, None) == -2
    assert step_ws(host, 0x1000, 0x2000, need, 1.5, 1e-3, 0.0, None) == -5
    assert step_ws(junk.ctypes.data, 0x1000, 0x2000, need, 0.9, 1e-3, 0.0, None) == -2
    assert fill(host, nbytes, T, M, n, xs, 0, gs, 0, None) == 0               # signSGD plan: no momentum
    assert step(host, 0x1000, 0.9, 1e-3, 0.0, None) == -5                     # momentum asked without v
    assert step_ws(host, 0x1000, 0x2000, need, 0.9, 1e-3, 0.0, None) == -5


def test_qsgd_argument_validation_needs_no_device(lib):
    P, W = 0x1000, 16
    lib.ssv_qsgd_workspace_bytes.restype = ctypes.c_size_t
    ws = lib.ssv_qsgd_workspace_bytes(3)
    assert ws > 0 and lib.ssv_qsgd_workspace_bytes(0) == 0 and lib.ssv_qsgd_workspace_bytes(1024) == 0
    assert lib.ssv_qsgd_workspace_bytes(6) == 2 * ws
    norms = lib.ssv_qsgd_norms
    norms.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert norms(None, 0, 3, 1000, 1000, 0, P, P, ws, None) == -1
    assert norms(P, 0, 3, 1000, 1000, 0, None, P, ws, None) == -1
    assert norms(P, 0, 3, 1000, 1000, 0, P, None, ws, None) == -1
    assert norms(P, 0, 3, 1000, 1000, 0, P, P, ws - 8, None) == -2          # workspace too small
    assert norms(P, 0, 3, 1000, 999, 0, P, P, ws, None) == -2
    assert norms(P, 0, 0, 1000, 1000, 0, P, P, ws, None) == -2
    assert norms(P, 3, 3, 1000, 1000, 0, P, P, ws, None) == -4
    assert norms(P, 0, 3, 1000, 1000, 2, P, P, ws, None) == -5              # unknown norm
    assert norms(P + 2, 0, 3, 1000, 1000, 0, P, P, ws, None) == -3
    assert norms(P, 0, 3, 1000, 1000, 0, P, P + 4, ws, None) == -3
    quant = lib.ssv_qsgd_quantize
    quant.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                      ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    assert quant(P, 0, None, P, 3, 1000, 1000, 1000, P, P, W, None) == -1
    assert quant(P, 0, P, P, 3, 1000, 1000, 1000, P, None, W, None) == -1
    assert quant(P, 0, P, P, 3, 1000, 1000, 999, P, P, W, None) == -2        # u rows shorter than d
    assert quant(P, 0, P, P, 3, 1000, 1000, 1000, P, P, W - 1, None) == -2
    assert quant(P, 5, P, P, 3, 1000, 1000, 1000, P, P, W, None) == -4
    assert quant(P, 0, P + 2, P, 3, 1000, 1000, 1000, P, P, W, None) == -3
    assert quant(P, 0, P, P, 3, 1000, 1000, 1000, P + 4, P, W, None) == -3
    agg = lib.ssv_qsgd_aggregate_apply
    agg.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_void_p]
    assert agg(None, P, P, 3, 1000, W, P, P, 0, 0.1, None) == -1
    assert agg(P, P, P, 3, 1000, W, None, None, 0, 0.1, None) == -1          # neither output
    assert agg(P, P, P, 3, 1000, W - 1, P, P, 0, 0.1, None) == -2
    assert agg(P, P, P, 3, 1000, W, P, P, 9, 0.1, None) == -4
    assert agg(P, P, P, 3, 1000, W, P, P, 0, float("nan"), None) == -5
    assert agg(P, P, P, 3, 1000, W, P + 2, P, 0, 0.1, None) == -3
    assert agg(P, P, P, 3, 1000, W, P, P + 1, 1, 0.1, None) == -3


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_1810_05291_amd as sv
    with pytest.raises(ValueError):
        sv.sign_pack(torch.zeros(2, 64))


def test_binding_checks_every_buffer_against_M_and_d_before_the_call():
    # shapes are validated before anything touches the device, so CPU tensors suffice to reach the checks:
    # a buffer that cannot hold M rows of d bits / d weights must never reach a kernel that would write past it
    import torch
    import paper_1810_05291_amd as sv
    M, d = 3, 1000
    W = sv.words_for(d)
    g = torch.zeros(M, d)
    v = torch.zeros(M, d)
    x = torch.zeros(d)
    rows = torch.zeros(M, W, dtype=torch.int64)
    vote = torch.zeros(W, dtype=torch.int64)

    def rejected(match, fn, *a, **k):
        with pytest.raises(ValueError, match=match):
            fn(*a, **k)

    # vote_apply: x shorter than d, d beyond the packed rows, short / mistyped vote_out
    rejected("x has", sv.vote_apply, rows, d, x[:-1], 1e-3)
    rejected("rows hold", sv.vote_apply, rows, 64 * W + 1, torch.zeros(64 * W + 1), 1e-3)
    rejected("vote_out holds", sv.vote_apply, rows, d, x, 1e-3, vote_out=vote[:-1])
    rejected("int64", sv.vote_apply, rows, d, x, 1e-3, vote_out=vote.to(torch.int32))
    rejected("int64", sv.vote_apply, rows.to(torch.int32), d, x, 1e-3)
    rejected("positive", sv.vote_apply, rows, 0, x, 1e-3)
    # apply_sign_update: vote must hold words_for(x.numel()) words
    rejected("vote holds", sv.apply_sign_update, x, vote[:-1], 1e-3)
    rejected("int64", sv.apply_sign_update, x, vote.to(torch.float64), 1e-3)
    rejected("contiguous", sv.apply_sign_update, torch.zeros(2 * d)[::2], vote, 1e-3)
    # majority_vote: d against the row width, vote size
    rejected("rows hold", sv.majority_vote, rows, 64 * W + 1)
    rejected("vote holds", sv.majority_vote, rows, d, vote[:-1])
    rejected("2-D", sv.majority_vote, vote, d)
    # sign_pack / signum_momentum_pack: a supplied signs buffer must have M rows of enough words
    rejected("rows, expected", sv.sign_pack, g, rows[:2])
    rejected("rows hold", sv.sign_pack, g, rows[:, :-1])
    rejected("rows hold", sv.signum_momentum_pack, g, v, 0.9, rows[:, :-1])
    rejected("v must be", sv.signum_momentum_pack, g, v[:2], 0.9)
    # signum_step: x, vote_out, signs_out, worker_flip
    rejected("x has", sv.signum_step, g, v, 0.9, x[:-1], 1e-3)
    rejected("vote_out holds", sv.signum_step, g, v, 0.9, x, 1e-3, vote_out=vote[:-1])
    rejected("contiguous", sv.signum_step, g, v, 0.9, x, 1e-3, vote_out=torch.zeros(2 * W, dtype=torch.int64)[::2])
    rejected("int64", sv.signum_step, g, v, 0.9, x, 1e-3, vote_out=vote.to(torch.int16))
    rejected("rows, expected", sv.signum_step, g, v, 0.9, x, 1e-3, signs_out=rows[:2])
    rejected("rows hold", sv.signum_step, g, v, 0.9, x, 1e-3, signs_out=rows[:, :-1])
    rejected("contiguous rows", sv.signum_step, g, v, 0.9, x, 1e-3, signs_out=torch.zeros(W, M, dtype=torch.int64).T)
    rejected("worker_flip", sv.signum_step, g, v, 0.9, x, 1e-3, worker_flip=[1, 0])
    # well-formed arguments get as far as the device check (and stop there: no CPU path exists)
    rejected("GPU memory only", sv.signum_step, g, v, 0.9, x, 1e-3, vote_out=vote, signs_out=rows)
    rejected("GPU memory only", sv.vote_apply, rows, d, x, 1e-3, vote_out=vote)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1810_05291_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no cpu fallback", ""), f


def test_flat_layout_offsets():
    from paper_1810_05291_amd import FlatLayout
    import torch
    lay = FlatLayout([(3, 5), (7,), (2, 2, 2), ()])
    assert lay.sizes == [15, 7, 8, 1] and lay.offsets == [0, 15, 22, 30] and lay.numel == 31
    assert lay.row_stride() == 32 and lay.row_stride(64) == 64
    flat = torch.arange(31, dtype=torch.float32)
    views = lay.views(flat)
    assert [tuple(v.shape) for v in views] == [(3, 5), (7,), (2, 2, 2), ()]
    assert views[1][0].item() == 15 and views[3].item() == 30
    views[2].zero_()
    assert flat[22:30].abs().sum().item() == 0 and flat[21].item() == 21    # views alias the flat buffer
    with pytest.raises(ValueError):
        lay.views(torch.zeros(30))
