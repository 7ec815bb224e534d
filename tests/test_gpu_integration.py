"""GPU integration checks around the C ABI: caller streams, HIP graph replay, and the paper's toy
problem driven end to end through the fused step."""
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
    sv_.load_library()
    return sv_


def _host(t):
    return np.ascontiguousarray(wl.to_numpy(t.contiguous()))


def test_calls_follow_the_callers_stream(sv):
    # work enqueued on a side stream (default priority) is ordered with that stream's other work
    M, d = 7, 300_001
    g = wl.gaussian((M, d), 1.0, seed=1, device=DEV)
    x = wl.gaussian((d,), 0.02, seed=2, device=DEV)
    x_ref = _host(x).copy()
    side = torch.cuda.Stream(device=DEV)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        signs = sv.sign_pack(g)
        vote = sv.majority_vote(signs, d)
        sv.apply_sign_update(x, vote, 1e-3)
        sv.vote_apply(signs, d, x, 1e-3)
    side.synchronize()
    ora.signum_step(_host(g), None, 0.0, x_ref, 1e-3)
    ora.signum_step(_host(g), None, 0.0, x_ref, 1e-3)
    assert np.array_equal(_host(x), x_ref)


def test_bench_copy_copies(sv):
    src = wl.gaussian((1_000_000,), 1.0, seed=8, device=DEV)
    dst = torch.zeros(1_000_004, device=DEV)
    sv.bench_copy(src, dst[:1_000_000])
    torch.cuda.synchronize()
    assert torch.equal(dst[:1_000_000], src) and (dst[1_000_000:] == 0).all()
    with pytest.raises(sv.SignvoteError):
        sv.bench_copy(src[1:5], dst[1:5])            # not 16-byte aligned


@pytest.mark.parametrize("with_signs", [False, True])
def test_fused_step_replays_in_a_hip_graph(sv, with_signs):
    # the library only launches kernels (no allocation, no memset), so a call can be captured;
    # every replay is one more optimiser step and must match eager execution bit for bit.
    # with_signs: the call is given room for the packed signs and runs as two kernels, both captured.
    M, d = 15, 200_003
    mu = wl.shared_mean(d, seed=3, device=DEV)
    g = wl.worker_gradients(mu, M, 0, base_seed=40)
    x_g = wl.gaussian((d,), 0.02, seed=5, device=DEV)
    v_g = torch.zeros((M, d), device=DEV)
    x_e, v_e = x_g.clone(), v_g.clone()
    vote_g = torch.zeros((sv.words_for(d),), dtype=torch.int64, device=DEV)
    vote_e = torch.zeros_like(vote_g)
    signs_g = torch.zeros((M, sv.words_for(d)), dtype=torch.int64, device=DEV) if with_signs else None
    signs_e = None if signs_g is None else torch.zeros_like(signs_g)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream(device=DEV)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sv.signum_step(g, v_g, 0.9, x_g, 1e-4, vote_out=vote_g, signs_out=signs_g)
    torch.cuda.synchronize()
    # capture does not execute: state is still the initial one
    assert torch.equal(x_g, x_e) and torch.equal(v_g, v_e)
    x_ref, v_ref = _host(x_e).copy(), np.zeros((M, d), np.float32)
    g_h = _host(g)
    for step in range(4):
        graph.replay()
        sv.signum_step(g, v_e, 0.9, x_e, 1e-4, vote_out=vote_e, signs_out=signs_e)       # eager work between replays
        torch.cuda.synchronize()
        vote_ref, signs_ref = ora.signum_step(g_h, v_ref, 0.9, x_ref, 1e-4, want_signs=True)
        assert torch.equal(x_g, x_e) and torch.equal(v_g, v_e) and torch.equal(vote_g, vote_e), f"replay {step}"
        assert np.array_equal(_host(x_g), x_ref) and np.array_equal(_host(vote_g), vote_ref)
        if with_signs:
            assert torch.equal(signs_g, signs_e) and np.array_equal(_host(signs_g), signs_ref)


def _quadratic_run(sv, M, adversaries, steps, mode, seed):
    """signSGD with majority vote on f(x) = |x|^2 / 2 in 1000 dimensions, N(0,1) noise on every
    gradient component (the paper's toy experiment, first figure); returns the loss curve and checks the
    trajectory against the oracle at every step."""
    d, lr = 1000, 1e-2
    x = wl.gaussian((d,), 1.0, seed=seed, device=DEV)
    x_ref = _host(x).copy()
    flip = [1] * adversaries + [0] * (M - adversaries)
    losses = [float(0.5 * (x_ref.astype(np.float64) ** 2).sum())]
    for k in range(steps):
        noise = wl.gaussian((M, d), 1.0, seed=seed + 1 + k, device=DEV)
        g = (x[None, :] + noise).contiguous()                       # gradient of the quadratic is x
        # the oracle runs its own closed loop: its gradient comes from ITS weights plus the same noise
        g_h = (x_ref[None, :] + _host(noise)).astype(np.float32)
        if mode == "invert":
            sv.signum_step(g, None, 0.0, x, lr, worker_flip=flip)
            ora.signum_step(g_h, None, 0.0, x_ref, lr, worker_flip=flip)
        else:                                                        # adversaries send random signs
            signs = sv.sign_pack(g)
            rnd = wl.random_words((adversaries, signs.shape[1]), seed=seed + 10_000 + k, device=DEV)
            signs[:adversaries] = rnd
            sv.vote_apply(signs, d, x, lr)
            s_h = ora.sign_pack(g_h)
            s_h[:adversaries] = _host(rnd)
            ora.vote_apply(s_h, d, x_ref, lr)
        torch.cuda.synchronize()
        assert np.array_equal(_host(x), x_ref), f"trajectory left the oracle's at step {k}"
        losses.append(float(0.5 * (x_ref.astype(np.float64) ** 2).sum()))
    return losses


def test_toy_quadratic_converges_and_degrades_gracefully(sv):
    M, steps = 27, 300
    clean = _quadratic_run(sv, M, 0, steps, "invert", seed=100)
    some = _quadratic_run(sv, M, 9, steps, "invert", seed=100)        # a third of the workers invert
    many = _quadratic_run(sv, M, 13, steps, "invert", seed=100)       # 48%: still a (thin) honest majority
    rnd = _quadratic_run(sv, M, 13, steps, "random", seed=100)
    print(f"toy quadratic, loss after {steps} steps from {clean[0]:.1f}: no adversaries {clean[-1]:.2f}, "
          f"9/27 inverting {some[-1]:.2f}, 13/27 inverting {many[-1]:.2f}, 13/27 random {rnd[-1]:.2f}", flush=True)
    assert clean[-1] < 0.05 * clean[0]
    assert some[-1] < 0.2 * some[0]
    assert many[-1] < many[0]                      # still descends with 48% adversaries
    assert rnd[-1] < 0.2 * rnd[0]                  # random adversaries hurt less than inverting ones
    assert clean[-1] <= some[-1] <= many[-1]
    # with an adversarial majority the vote points uphill
    lost = _quadratic_run(sv, M, 14, 60, "invert", seed=100)
    assert lost[-1] > lost[0]


_VARIANT_SCRIPT = r"""
import numpy as np, torch, sys
sys.path.insert(0, %r)
import paper_1810_05291_amd as sv, oracle as ora, workloads as wl
dev = "cuda:0"
for (M, d, gdt) in ((15, 100_003, torch.float32), (31, 70_001, torch.bfloat16), (3, 17, torch.float32)):
    mu = wl.shared_mean(d, seed=1, device=dev)
    x = wl.gaussian((d,), 0.02, seed=2, device=dev)
    v = torch.zeros((M, d), device=dev)
    x_ref, v_ref = wl.to_numpy(x).copy(), np.zeros((M, d), np.float32)
    W = sv.words_for(d)
    for step in range(2):
        g = wl.worker_gradients(mu, M, step, base_seed=9, dtype=gdt)
        vote = torch.empty((W,), dtype=torch.int64, device=dev)
        signs = torch.empty((M, W), dtype=torch.int64, device=dev)
        sv.signum_step(g, v, 0.9, x, 1e-4, vote_out=vote, signs_out=signs)
        x2 = x.clone(); sv.vote_apply(signs, d, x2, 1e-4)
        torch.cuda.synchronize()
        vote_ref, signs_ref = ora.signum_step(wl.to_numpy(g), v_ref, 0.9, x_ref, 1e-4, want_signs=True)
        assert np.array_equal(wl.to_numpy(signs), signs_ref) and np.array_equal(wl.to_numpy(vote), vote_ref)
        assert np.array_equal(wl.to_numpy(v), v_ref) and np.array_equal(wl.to_numpy(x), x_ref)
        x_ref2 = x_ref.copy(); ora.apply_sign_update(x_ref2, vote_ref, 1e-4)
        assert np.array_equal(wl.to_numpy(x2), x_ref2)
        sv.signum_step(g, v, 0.9, x, 1e-4)                    # lean form
        torch.cuda.synchronize()
        ora.signum_step(wl.to_numpy(g), v_ref, 0.9, x_ref, 1e-4)
        assert np.array_equal(wl.to_numpy(v), v_ref) and np.array_equal(wl.to_numpy(x), x_ref)
print("variant ok")
"""


@pytest.mark.parametrize("env", [{"SSV_TUNE_STEP_SERIAL": "0"}])
def test_measurement_switch_keeps_parity(env):
    # SSV_TUNE_STEP_SERIAL is read once per process, so the non-default setting runs in a child process
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    child_env = dict(os.environ, **env)
    r = subprocess.run([sys.executable, "-c", _VARIANT_SCRIPT % root], env=child_env, capture_output=True, text=True,
                       timeout=240)
    assert r.returncode == 0 and "variant ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]


def test_small_model_trains_through_the_flat_layout(sv):
    # a two-layer network on synthetic regression data, 5 simulated workers with their own mini-batches;
    # many parameter tensors, one flat vector, one launch per step.  The gradients (torch autograd) are the
    # recorded inputs of each step; the oracle is fed the same recorded gradients and must land on the same
    # weights and momenta.
    torch.manual_seed(0)
    M, steps = 5, 60
    shapes = [(64, 20), (64,), (1, 64), (1,)]
    opt = sv.SignumMajorityVote(shapes, M, lr=2e-3, beta=0.9, device=DEV)
    for p, std in zip(opt.params, (0.2, 0.0, 0.1, 0.0)):
        p.copy_(torch.randn(p.shape, device=DEV) * std)
    params = [p.detach().requires_grad_() for p in opt.params]        # leaves that alias the flat vector
    w_true = torch.randn(20, device=DEV)

    def batch(seed, n=64):
        gen = torch.Generator(device=DEV).manual_seed(seed)
        xb = torch.randn(n, 20, device=DEV, generator=gen)
        yb = torch.tanh(xb @ w_true)[:, None] + 0.05 * torch.randn(n, 1, device=DEV, generator=gen)
        return xb, yb

    def loss_fn(xb, yb):
        h = torch.relu(xb @ params[0].T + params[1])
        return ((h @ params[2].T + params[3] - yb) ** 2).mean()

    x_ref = _host(opt.x).copy()
    v_ref = np.zeros((M, opt.layout.numel), np.float32)
    xe, ye = batch(10_000, 2048)
    first = loss_fn(xe, ye).item()
    for k in range(steps):
        for m in range(M):
            grads = torch.autograd.grad(loss_fn(*batch(1 + k * M + m)), params)
            for dst, src in zip(opt.grads[m], grads):
                dst.copy_(src)
        opt.step()
        torch.cuda.synchronize()
        ora.signum_step(_host(opt.g), v_ref, 0.9, x_ref, 2e-3)
        assert np.array_equal(_host(opt.x), x_ref), f"step {k}"
    assert np.array_equal(_host(opt.v), v_ref)
    last = loss_fn(xe, ye).item()
    print(f"small model: evaluation loss {first:.4f} -> {last:.4f} in {steps} fused steps", flush=True)
    assert last < 0.5 * first
    # checkpoint / resume: state is x, the momenta and the step count
    state = opt.state_dict()
    opt.step()
    after = opt.x.clone()
    opt.load_state_dict(state)
    opt.step()
    assert torch.equal(opt.x, after)


@pytest.mark.parametrize("driver", ["flat", "multi"])
def test_drivers_replay_their_step_as_a_hip_graph(sv, driver):
    # capture_graph() records one step (two kernel launches) once; every later step() is a replay.  Replays are
    # interleaved with eager work and synchronisations and compared with an eager twin and with the oracle.
    M, steps = 4, 6
    shapes = [(33, 7), (33,), (5000,), (1,)]
    sizes = [int(np.prod(s)) for s in shapes]
    if driver == "flat":
        make = lambda: sv.SignumMajorityVote(shapes, M, lr=1e-3, beta=0.9, device=DEV)
        graphed, eager = make(), make()
        grads_of = lambda o: o.grads
        weights_of = lambda o: [p.reshape(-1) for p in o.params]
    else:
        def make():
            params = [torch.zeros(s, device=DEV) for s in shapes]
            wg = [[torch.zeros(s, device=DEV) for s in shapes] for _ in range(M)]
            return sv.SignumMajorityVoteMulti(params, wg, lr=1e-3, beta=0.9)
        graphed, eager = make(), make()
        grads_of = lambda o: o.worker_grads
        weights_of = lambda o: [p.reshape(-1) for p in o.params]
    for o in (graphed, eager):
        for t, w in enumerate(weights_of(o)):
            w.copy_(wl.gaussian((sizes[t],), 0.02, seed=50 + t, device=DEV))
    x_ref = [_host(w).copy() for w in weights_of(eager)]
    v_ref = [np.zeros((M, n), np.float32) for n in sizes]
    graphed.capture_graph()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(weights_of(graphed), weights_of(eager))), "capture must not execute"
    for k in range(steps):
        for t, n in enumerate(sizes):
            gt = wl.gaussian((M, n), 1e-2, seed=900 + 10 * k + t, device=DEV)
            for o in (graphed, eager):
                for m in range(M):
                    grads_of(o)[m][t].reshape(-1).copy_(gt[m])
            ora.signum_step(_host(gt), v_ref[t], 0.9, x_ref[t], 1e-3)
        graphed.step()                                          # replay
        eager.step()                                            # eager launches between the replays
        torch.cuda.synchronize()
        for t in range(len(sizes)):
            assert torch.equal(weights_of(graphed)[t], weights_of(eager)[t]), f"replay {k}, tensor {t}"
            assert np.array_equal(_host(weights_of(graphed)[t]), x_ref[t]), f"replay {k}, tensor {t} vs the oracle"
    assert graphed.steps == steps


def test_small_model_trains_with_gradients_left_where_autograd_put_them(sv):
    # the same two-layer network, but every worker's gradients stay in the tensors autograd wrote them to; the
    # multi-tensor step takes them from there (no copy into a flat buffer), one launch per step
    torch.manual_seed(0)
    M, steps = 5, 60
    shapes = [(64, 20), (64,), (1, 64), (1,)]
    stds = (0.2, 0.0, 0.1, 0.0)
    params = [(torch.randn(s, device=DEV) * std).requires_grad_() for s, std in zip(shapes, stds)]
    worker_grads = [[torch.zeros(s, device=DEV) for s in shapes] for _ in range(M)]
    opt = sv.SignumMajorityVoteMulti([p.detach() for p in params], worker_grads, lr=2e-3, beta=0.9)
    w_true = torch.randn(20, device=DEV)

    def batch(seed, n=64):
        gen = torch.Generator(device=DEV).manual_seed(seed)
        xb = torch.randn(n, 20, device=DEV, generator=gen)
        yb = torch.tanh(xb @ w_true)[:, None] + 0.05 * torch.randn(n, 1, device=DEV, generator=gen)
        return xb, yb

    def loss_fn(xb, yb):
        h = torch.relu(xb @ params[0].T + params[1])
        return ((h @ params[2].T + params[3] - yb) ** 2).mean()

    x_ref = [_host(p.detach()).reshape(-1).copy() for p in params]
    v_ref = [np.zeros((M, p.numel()), np.float32) for p in params]
    xe, ye = batch(10_000, 2048)
    first = loss_fn(xe, ye).item()
    for k in range(steps):
        for m in range(M):
            for t, p in enumerate(params):
                p.grad = worker_grads[m][t]                         # autograd accumulates into the worker's own tensors
                p.grad.zero_()
            loss_fn(*batch(1 + k * M + m)).backward()
        opt.step()
        torch.cuda.synchronize()
        for t, p in enumerate(params):
            g_h = np.stack([_host(worker_grads[m][t]).reshape(-1) for m in range(M)])
            ora.signum_step(g_h, v_ref[t], 0.9, x_ref[t], 2e-3)
            assert np.array_equal(_host(p.detach()).reshape(-1), x_ref[t]), f"tensor {t}, step {k}"
    last = loss_fn(xe, ye).item()
    print(f"small model, multi-tensor step: evaluation loss {first:.4f} -> {last:.4f} in {steps} fused steps", flush=True)
    assert last < 0.5 * first
