"""Plumbing for real models with many parameter tensors: the tensor fusion that Section 4 of the paper
credits with a speed-up of compression and communication.  Two ways to get one library call per step (two
kernel launches: pack row by row, then vote + update) however many tensors the model has:

SignumMajorityVote       lays the tensors out back to back in ONE flat buffer, once, and hands out views for
                         the parameters and for each simulated worker's gradients.  The step itself copies
                         nothing -- but whoever produces the gradients must write them into those views; a
                         model whose autograd leaves gradients in tensors of its own pays one copy per
                         worker per step to move them there.
SignumMajorityVoteMulti  takes the weight tensors and every worker's gradient tensors where they are (a table
                         of device addresses, built once) and runs the step over the concatenated index
                         space with per-tensor ragged ends: no copy at all.

Only memory plumbing lives here; all arithmetic is in libsignvote.
"""
import math

import torch

from . import binding as _b


class FlatLayout:
    """Offsets of a list of tensor shapes inside one flat vector (back to back, no padding: the
    kernels handle any d, and padding coordinates would be updated like real ones)."""

    def __init__(self, shapes):
        self.shapes = [tuple(int(s) for s in shape) for shape in shapes]
        self.sizes = [int(math.prod(s)) for s in self.shapes]
        self.offsets = []
        off = 0
        for n in self.sizes:
            self.offsets.append(off)
            off += n
        self.numel = off
        if self.numel < 1:
            raise ValueError("empty layout")

    def row_stride(self, align_elems=32):
        """Row stride for [M][stride] buffers: numel rounded up so that every row starts on a 128-byte boundary."""
        return ((self.numel + align_elems - 1) // align_elems) * align_elems

    def views(self, flat):
        """One view per tensor into the 1-D buffer `flat` (at least numel elements)."""
        if flat.dim() != 1 or flat.numel() < self.numel:
            raise ValueError("flat buffer too small")
        return [flat[o:o + n].view(s) for o, n, s in zip(self.offsets, self.sizes, self.shapes)]


class _GraphedStep:
    """Optional HIP graph around a driver's step: the library only launches kernels on the caller's stream (no
    allocation, no memset), so one step can be captured once and replayed.  For small models the two launches of a
    step cost more on the host than on the GPU; a replay is one host call."""

    _graph = None

    def capture_graph(self):
        """Capture one step into a HIP graph; from then on step() without arguments replays it.  The buffers the
        step reads and writes keep their addresses for the life of the driver, so replays see refilled gradients."""
        dev = self._graph_device()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream(device=dev)
        side.wait_stream(torch.cuda.current_stream(dev))
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                self._launch()
        torch.cuda.current_stream(dev).wait_stream(side)
        self._graph = graph                                   # capture does not execute: no step has been taken


class SignumMajorityVote(_GraphedStep):
    """Signum with majority vote (Algorithm 1) for M simulated workers on one GPU.

    params            list of views into the flat weight vector (update happens in place)
    grads[m]          list of views into worker m's flat gradient row: write gradients there
    step()            one library call: momentum, sign, vote, update for all workers
    """

    def __init__(self, shapes, num_workers, lr=1e-4, beta=0.9, weight_decay=0.0, device="cuda:0",
                 param_dtype=torch.float32, grad_dtype=torch.float32):
        if num_workers < 1:
            raise ValueError("need at least one worker")
        self.layout = FlatLayout(shapes)
        self.M = int(num_workers)
        self.lr, self.beta, self.weight_decay = float(lr), float(beta), float(weight_decay)
        d = self.layout.numel
        stride_g = self.layout.row_stride(32 if grad_dtype == torch.float32 else 64)
        stride_v = self.layout.row_stride(32)
        self.x = torch.zeros((d,), dtype=param_dtype, device=device)
        self.g = torch.zeros((self.M, stride_g), dtype=grad_dtype, device=device)[:, :d]
        self.v = torch.zeros((self.M, stride_v), dtype=torch.float32, device=device)[:, :d] if self.beta > 0 else None
        self.params = self.layout.views(self.x)
        self.grads = [self.layout.views(self.g[m]) for m in range(self.M)]
        # room for what the workers transmit (M * d / 8 bytes): with it the library runs the step in its fastest form
        W = _b.words_for(d)
        self.signs = torch.empty((self.M, ((W + 15) // 16) * 16), dtype=torch.int64, device=device)[:, :W]
        self.steps = 0

    def _graph_device(self):
        return self.x.device

    def _launch(self, worker_flip=None, vote_out=None):
        _b.signum_step(self.g, self.v, self.beta, self.x, self.lr, self.weight_decay, vote_out=vote_out,
                       signs_out=self.signs, worker_flip=worker_flip)

    def step(self, worker_flip=None, vote_out=None):
        if self._graph is not None and worker_flip is None and vote_out is None:
            self._graph.replay()
        else:
            self._launch(worker_flip, vote_out)
        self.steps += 1

    def state_dict(self):
        """Everything Algorithm 1 carries between iterations: x, the per-worker momenta, the step count."""
        return {"x": self.x.clone(), "v": None if self.v is None else self.v.clone(), "steps": self.steps}

    def load_state_dict(self, state):
        self.x.copy_(state["x"])
        if self.v is not None:
            self.v.copy_(state["v"])
        self.steps = int(state["steps"])


class SignumMajorityVoteMulti(_GraphedStep):
    """Signum with majority vote (Algorithm 1) on tensors that stay where they are.

    params          list of T weight tensors on the GPU (updated in place)
    worker_grads    M lists of T gradient tensors (worker m's gradient of tensor t); the same tensor objects
                    must be refilled in place every step (their addresses are in the plan)
    Momenta (fp32) are allocated here, one 128-byte aligned slice per tensor in one buffer per worker.
    step()          one library call over all tensors
    """

    def __init__(self, params, worker_grads, lr=1e-4, beta=0.9, weight_decay=0.0):
        self.params = list(params)
        self.worker_grads = [list(row) for row in worker_grads]
        self.M = len(self.worker_grads)
        self.lr, self.beta, self.weight_decay = float(lr), float(beta), float(weight_decay)
        self.momenta = None
        if self.beta > 0:
            offs, off = [], 0
            for p in self.params:
                offs.append(off)
                off += ((p.numel() + 31) // 32) * 32
            dev = self.params[0].device
            self._vbuf = torch.zeros((self.M, max(off, 32)), dtype=torch.float32, device=dev)
            self.momenta = [[self._vbuf[m, o:o + p.numel()] for o, p in zip(offs, self.params)] for m in range(self.M)]
        self.plan = _b.MultiTensorPlan(self.params, self.worker_grads, self.momenta)
        self.workspace = _b.multi_workspace(self.plan)      # the workers' packed signs: selects the two-kernel form
        self.steps = 0

    def _graph_device(self):
        return self.params[0].device

    def _launch(self):
        _b.signum_step_multi(self.plan, self.beta, self.lr, self.weight_decay, workspace=self.workspace)

    def step(self):
        if self._graph is not None:
            self._graph.replay()
        else:
            self._launch()
        self.steps += 1
