"""Seeded input generators (see the package docstring).  No arithmetic of the method lives here."""
import numpy as np
import torch

RESNET50_D = 25_557_032   # parameter count of the resnet50 the paper trains on ImageNet
LARGE_D = 1_500_000_000
STRESS_D = 1 << 30


def words_for(d: int) -> int:
    """64-bit words needed for d one-bit entries."""
    return (int(d) + 63) // 64


def _gen(seed: int, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def gaussian(shape, std: float, seed: int, device="cpu", dtype=torch.float32, out=None):
    """N(0, std) entries, i.i.d., from `seed`."""
    g = _gen(seed, device)
    if out is None:
        out = torch.empty(shape, device=device, dtype=torch.float32)
    assert out.dtype == torch.float32
    out.normal_(0.0, float(std), generator=g)
    return out if dtype == torch.float32 else out.to(dtype)


def tiny_config(seed: int = 0, device="cpu", d: int = 65_536, M: int = 3):
    """Config 'tiny': N(0,1) gradients for M workers and N(0, 0.02) weights."""
    g = gaussian((M, d), 1.0, seed, device)
    x = gaussian((d,), 0.02, seed + 7919, device)
    return g, x


def shared_mean(d: int, seed: int, device="cpu", std: float = 1e-3):
    """The fixed 'true gradient' mu of a run."""
    return gaussian((d,), std, seed, device)


def worker_gradients(mu, M: int, step: int, base_seed: int, noise_std: float = 1e-2, out=None,
                     dtype=torch.float32, row_stride=None):
    """g[m] = mu + N(0, noise_std), worker m at step k seeded with base_seed + 1000*k + m.

    Returns a [M, d] tensor (a view of a [M, row_stride] buffer when row_stride is given)."""
    d = mu.numel()
    stride = d if row_stride is None else int(row_stride)
    assert stride >= d
    if out is None:
        out = torch.empty((M, stride), device=mu.device, dtype=dtype)
    rows = out[:, :d]
    tmp = torch.empty((d,), device=mu.device, dtype=torch.float32)
    for m in range(M):
        gaussian((d,), noise_std, base_seed + 1000 * step + m, mu.device, out=tmp)
        tmp.add_(mu.to(torch.float32))
        rows[m].copy_(tmp)  # rounds to bf16 when the buffer is bf16
    return rows


def resnet50_parameter_shapes():
    """Shapes of the 161 parameter tensors of the 50-layer residual network the paper trains on ImageNet
    (bottleneck blocks [3, 4, 6, 3] of widths 64..512 with 4x expansion, batch-norm scale and shift after every
    convolution, a 1000-way linear classifier): 25,557,032 parameters in tensors of 64 .. 2,359,296 elements."""
    shapes = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            shapes += [(planes, inplanes, 1, 1), (planes,), (planes,),
                       (planes, planes, 3, 3), (planes,), (planes,),
                       (4 * planes, planes, 1, 1), (4 * planes,), (4 * planes,)]
            if b == 0:                                   # projection shortcut of the first block of a stage
                shapes += [(4 * planes, inplanes, 1, 1), (4 * planes,), (4 * planes,)]
            inplanes = 4 * planes
    shapes += [(1000, 2048), (1000,)]
    assert sum(int(np.prod(s)) for s in shapes) == RESNET50_D and len(shapes) == 161
    return shapes


def random_words(shape, seed: int, device="cpu"):
    """Uniform random 64-bit patterns (int64 storage): fair, independent sign bits."""
    g = _gen(seed, device)
    return torch.randint(-(1 << 63), (1 << 63) - 1, shape, generator=g, device=device, dtype=torch.int64)


def bernoulli_packed_rows(M: int, d: int, seed: int, device="cpu", lo: float = 0.3, hi: float = 0.7,
                          chunk_words: int = 1 << 14, out=None, row_stride_words=None):
    """Pre-packed sign rows for the vote stress test: bit(m, j) = [u(m,j) < p_j], p_j ~ U(lo, hi).

    Entry j sits at bit (j % 64) of word j // 64 (bit 0 = least significant); bits past d are 0.
    Returns (rows int64 [M, W] view, p float32 [d])."""
    W = words_for(d)
    stride = W if row_stride_words is None else int(row_stride_words)
    if out is None:
        out = torch.zeros((M, stride), device=device, dtype=torch.int64)
    rows = out[:, :W]
    g = _gen(seed, device)
    p = torch.empty((d,), device=device, dtype=torch.float32).uniform_(lo, hi, generator=g)
    weights = (torch.ones(64, dtype=torch.int64, device=device) << torch.arange(64, device=device))
    rows_per_pass = max(1, (1 << 26) // (chunk_words * 64))
    for w0 in range(0, W, chunk_words):
        w1 = min(W, w0 + chunk_words)
        n = (w1 - w0) * 64
        pj = torch.full((n,), -1.0, device=device)     # past-the-end entries never fire
        j1 = min(d, w1 * 64)
        pj[: j1 - w0 * 64] = p[w0 * 64: j1]
        for m0 in range(0, M, rows_per_pass):
            m1 = min(M, m0 + rows_per_pass)
            u = torch.rand((m1 - m0, n), device=device, generator=g)
            bits = (u < pj).view(m1 - m0, w1 - w0, 64).to(torch.int64)
            rows[m0:m1, w0:w1] = (bits * weights).sum(dim=2)
    return rows, p


def special_values_f32():
    """Edge-case floats for the sign convention: zeros, denormals, infinities, NaN."""
    tiny = np.float32(1e-45)            # smallest positive denormal
    mn = np.finfo(np.float32).tiny      # smallest positive normal
    return np.array([0.0, -0.0, tiny, -tiny, mn, -mn, 1.0, -1.0, np.inf, -np.inf, np.nan,
                     3.4e38, -3.4e38], dtype=np.float32)


def to_numpy(t):
    """Host numpy copy; bf16 tensors come back as uint16 bit patterns, int64 words as uint64."""
    t = t.detach()
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    a = t.cpu().numpy()
    if a.dtype == np.int64:
        return a.view(np.uint64)
    return a


def bf16_bits(t):
    return to_numpy(t.to(torch.bfloat16))
