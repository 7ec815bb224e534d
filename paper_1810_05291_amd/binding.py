"""ctypes binding of libsignvote.so: same names as the C ABI, argument marshalling only.

Tensors must live on the GPU.  Packed sign rows are torch.int64 tensors (bit patterns of the
uint64 words).  Every call is enqueued on torch's current stream of the tensors' device and
returns without synchronising.
"""
import ctypes
import os

import torch

SSV_F32 = 0
SSV_BF16 = 1
SSV_QSGD_L2 = 0
SSV_QSGD_MAX = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

_c_i64 = ctypes.c_int64
_c_int = ctypes.c_int
_c_f = ctypes.c_float
_c_p = ctypes.c_void_p

_SIGNATURES = {
    "ssv_sign_pack": [_c_p, _c_int, _c_int, _c_i64, _c_i64, _c_p, _c_i64, _c_p],
    "ssv_signum_momentum_pack": [_c_p, _c_int, _c_p, _c_int, _c_i64, _c_i64, _c_i64, _c_f, _c_p, _c_i64, _c_p],
    "ssv_majority_vote": [_c_p, _c_int, _c_i64, _c_i64, _c_p, _c_p],
    "ssv_apply_sign_update": [_c_p, _c_int, _c_i64, _c_p, _c_f, _c_f, _c_p],
    "ssv_vote_apply": [_c_p, _c_int, _c_i64, _c_i64, _c_p, _c_int, _c_f, _c_f, _c_p, _c_p],
    "ssv_signum_step": [_c_p, _c_int, _c_p, _c_int, _c_i64, _c_i64, _c_i64, _c_f, _c_p, _c_int, _c_f, _c_f,
                        _c_p, _c_p, _c_i64, _c_p, _c_p],
    "ssv_bench_copy": [_c_p, _c_p, _c_i64, _c_p],
}


class SignvoteError(RuntimeError):
    def __init__(self, name, status):
        self.status = int(status)
        super().__init__(f"{name} failed with status {status}: {status_string(status)}")


def library_path() -> str:
    return os.environ.get("SIGNVOTE_LIB", os.path.join(_HERE, "libsignvote.so"))


def load_library():
    """Load libsignvote.so (built in-tree).  Raises ImportError if it is missing: there is no fallback."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} not found: build it with `python -m paper_1810_05291_amd.build`")
        lib = ctypes.CDLL(path)
        for name, argtypes in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.argtypes = argtypes
            fn.restype = _c_int
        lib.ssv_multi_plan_bytes.argtypes = [_c_int, _c_int, _c_p]
        lib.ssv_multi_plan_bytes.restype = ctypes.c_size_t
        lib.ssv_multi_plan_fill.argtypes = [_c_p, ctypes.c_size_t, _c_int, _c_int, _c_p, _c_p, _c_int, _c_p, _c_int, _c_p]
        lib.ssv_multi_plan_fill.restype = _c_int
        lib.ssv_signum_step_multi.argtypes = [_c_p, _c_p, _c_f, _c_f, _c_f, _c_p]
        lib.ssv_signum_step_multi.restype = _c_int
        lib.ssv_multi_workspace_bytes.argtypes = [_c_p]
        lib.ssv_multi_workspace_bytes.restype = ctypes.c_size_t
        lib.ssv_signum_step_multi_ws.argtypes = [_c_p, _c_p, _c_p, ctypes.c_size_t, _c_f, _c_f, _c_f, _c_p]
        lib.ssv_signum_step_multi_ws.restype = _c_int
        lib.ssv_qsgd_workspace_bytes.argtypes = [_c_int]
        lib.ssv_qsgd_workspace_bytes.restype = ctypes.c_size_t
        lib.ssv_qsgd_norms.argtypes = [_c_p, _c_int, _c_int, _c_i64, _c_i64, _c_int, _c_p, _c_p, ctypes.c_size_t, _c_p]
        lib.ssv_qsgd_norms.restype = _c_int
        lib.ssv_qsgd_norms_static.argtypes = [_c_p, _c_int, _c_int, _c_i64, _c_i64, _c_int, _c_p, _c_p]
        lib.ssv_qsgd_norms_static.restype = _c_int
        lib.ssv_qsgd_quantize.argtypes = [_c_p, _c_int, _c_p, _c_p, _c_int, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_i64, _c_p]
        lib.ssv_qsgd_quantize.restype = _c_int
        lib.ssv_qsgd_aggregate_apply.argtypes = [_c_p, _c_p, _c_p, _c_int, _c_i64, _c_i64, _c_p, _c_p, _c_int, _c_f, _c_p]
        lib.ssv_qsgd_aggregate_apply.restype = _c_int
        lib.ssv_status_string.argtypes = [_c_int]
        lib.ssv_status_string.restype = ctypes.c_char_p
        lib.ssv_version.argtypes = []
        lib.ssv_version.restype = _c_int
        _LIB = lib
    return _LIB


def status_string(status: int) -> str:
    return load_library().ssv_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().ssv_version())


def words_for(d: int) -> int:
    return (int(d) + 63) // 64


def _dt(t):
    if t.dtype == torch.float32:
        return SSV_F32
    if t.dtype == torch.bfloat16:
        return SSV_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(*tensors):
    dev = None
    for t in tensors:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("libsignvote works on GPU memory only")
        if dev is None:
            dev = t.device
        elif t.device != dev:
            raise ValueError("all tensors must be on one device")
    return dev


def _rows(t):
    """(M, d, row stride in elements) of a 2-D tensor whose rows are contiguous."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a 2-D tensor with contiguous rows")
    return t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _vec(t):
    if t.dim() != 1 or (t.numel() > 1 and t.stride(0) != 1):
        raise ValueError("expected a contiguous 1-D tensor")
    return t


def _ptr(t):
    return None if t is None else t.data_ptr()


def _packed_rows(t, M, d, name):
    """Row stride (words) of a packed [M][>= ceil(d/64)] int64 tensor, after checking that it can hold M rows of d bits."""
    if t.dtype != torch.int64:
        raise ValueError(f"{name} must be torch.int64 (bit patterns of the packed words)")
    rows, cols, stride = _rows(t)
    if rows != M:
        raise ValueError(f"{name} has {rows} rows, expected {M}")
    if cols < words_for(d):
        raise ValueError(f"{name} rows hold {cols} words, {words_for(d)} needed for d = {d}")
    return stride


def _packed_vec(t, d, name):
    """A contiguous int64 vector of at least ceil(d/64) words."""
    if t.dtype != torch.int64:
        raise ValueError(f"{name} must be torch.int64 (bit patterns of the packed words)")
    if _vec(t).numel() < words_for(d):
        raise ValueError(f"{name} holds {t.numel()} words, {words_for(d)} needed for d = {d}")
    return t


def _weights(x, d):
    _dt(x)
    if _vec(x).numel() != d:
        raise ValueError(f"x has {x.numel()} elements, expected d = {d}")
    return x


def _dim(d):
    d = int(d)
    if d < 1:
        raise ValueError("d must be positive")
    return d


def _stream(dev):
    return torch.cuda.current_stream(dev).cuda_stream


def _check(name, rc):
    if rc != 0:
        raise SignvoteError(name, rc)


def sign_pack(x, signs=None):
    """signs[m] = packed (x[m] >= 0) for every row of the 2-D tensor x."""
    M, d, xs = _rows(x)
    ss = None if signs is None else _packed_rows(signs, M, d, "signs")
    dev = _dev(x, signs)
    if signs is None:
        signs = torch.empty((M, words_for(d)), dtype=torch.int64, device=dev)
        ss = words_for(d)
    _check("ssv_sign_pack", load_library().ssv_sign_pack(_ptr(x), _dt(x), M, d, xs, _ptr(signs), ss, _stream(dev)))
    return signs


def signum_momentum_pack(g, v, beta, signs=None):
    """v <- (1-beta) g + beta v in place; returns packed signs of the new v."""
    M, d, gs = _rows(g)
    Mv, dv, vs = _rows(v)
    if (Mv, dv) != (M, d) or v.dtype != torch.float32:
        raise ValueError("v must be fp32 with the shape of g")
    ss = None if signs is None else _packed_rows(signs, M, d, "signs")
    dev = _dev(g, v, signs)
    if signs is None:
        signs = torch.empty((M, words_for(d)), dtype=torch.int64, device=dev)
        ss = words_for(d)
    _check("ssv_signum_momentum_pack",
           load_library().ssv_signum_momentum_pack(_ptr(g), _dt(g), _ptr(v), M, d, gs, vs, float(beta), _ptr(signs),
                                                   ss, _stream(dev)))
    return signs


def majority_vote(signs, d, vote=None):
    """Packed element-wise majority over the rows of `signs` (ties -> +1)."""
    d = _dim(d)
    M = signs.shape[0] if signs.dim() == 2 else 0
    ss = _packed_rows(signs, M, d, "signs")
    if vote is not None:
        _packed_vec(vote, d, "vote")
    dev = _dev(signs, vote)
    if vote is None:
        vote = torch.empty((words_for(d),), dtype=torch.int64, device=dev)
    _check("ssv_majority_vote", load_library().ssv_majority_vote(_ptr(signs), M, d, ss, _ptr(vote), _stream(dev)))
    return vote


def apply_sign_update(x, vote, lr, weight_decay=0.0):
    """x <- x - lr (vote + weight_decay x) in place."""
    d = _dim(x.numel())
    _weights(x, d)
    _packed_vec(vote, d, "vote")
    dev = _dev(x, vote)
    _check("ssv_apply_sign_update",
           load_library().ssv_apply_sign_update(_ptr(x), _dt(x), d, _ptr(vote), float(lr), float(weight_decay),
                                                _stream(dev)))
    return x


def vote_apply(signs, d, x, lr, weight_decay=0.0, vote_out=None):
    """Fused majority vote + update from packed rows."""
    d = _dim(d)
    M = signs.shape[0] if signs.dim() == 2 else 0
    ss = _packed_rows(signs, M, d, "signs")
    _weights(x, d)
    if vote_out is not None:
        _packed_vec(vote_out, d, "vote_out")
    dev = _dev(signs, x, vote_out)
    _check("ssv_vote_apply",
           load_library().ssv_vote_apply(_ptr(signs), M, d, ss, _ptr(x), _dt(x), float(lr), float(weight_decay),
                                         _ptr(vote_out), _stream(dev)))
    return x


def signum_step(g, v, beta, x, lr, weight_decay=0.0, vote_out=None, signs_out=None, worker_flip=None):
    """One fused iteration of Algorithm 1 for all workers.  v may be None (signSGD, beta = 0)."""
    M, d, gs = _rows(g)
    vs = 0
    if v is not None:
        Mv, dv, vs = _rows(v)
        if (Mv, dv) != (M, d) or v.dtype != torch.float32:
            raise ValueError("v must be fp32 with the shape of g")
    _weights(x, d)
    if vote_out is not None:
        _packed_vec(vote_out, d, "vote_out")
    ss = 0 if signs_out is None else _packed_rows(signs_out, M, d, "signs_out")
    flip = None
    if worker_flip is not None:
        if len(worker_flip) != M:
            raise ValueError(f"worker_flip has {len(worker_flip)} entries, expected M = {M}")
        flip = (ctypes.c_uint8 * M)(*[1 if f else 0 for f in worker_flip])
    dev = _dev(g, v, x, vote_out, signs_out)
    _check("ssv_signum_step",
           load_library().ssv_signum_step(_ptr(g), _dt(g), _ptr(v), M, d, gs, vs, float(beta), _ptr(x), _dt(x),
                                          float(lr), float(weight_decay), _ptr(vote_out), _ptr(signs_out), ss,
                                          ctypes.cast(flip, _c_p) if flip is not None else None, _stream(dev)))
    return x


class MultiTensorPlan:
    """The plan of ssv_signum_step_multi for T weight tensors and M workers' gradient (and momentum) tensors.

    params[t]      weight tensor t (contiguous, fp32 or bf16, one dtype for all)
    grads[m][t]    worker m's gradient of tensor t (contiguous, same number of elements, one dtype for all)
    momenta[m][t]  worker m's fp32 momentum of tensor t, or momenta=None for signSGD
    The tensors are referenced (kept alive), not copied; the plan holds their addresses, so they must not be
    reallocated while the plan is in use.  The device copy of the plan is made here, once."""

    def __init__(self, params, grads, momenta=None):
        lib = load_library()
        T, M = len(params), len(grads)
        if T < 1 or M < 1:
            raise ValueError("need at least one tensor and one worker")
        if any(len(row) != T for row in grads) or (momenta is not None and
                                                  (len(momenta) != M or any(len(row) != T for row in momenta))):
            raise ValueError("grads and momenta must be M lists of T tensors")
        dev = _dev(*params, *[t for row in grads for t in row], *([t for row in momenta for t in row] if momenta else []))
        x_dt, g_dt = _dt(params[0]), _dt(grads[0][0])
        n = (ctypes.c_int64 * T)()
        xs = (ctypes.c_void_p * T)()
        gs = (ctypes.c_void_p * (T * M))()
        vs = (ctypes.c_void_p * (T * M))() if momenta is not None else None
        for t, p in enumerate(params):
            if not p.is_contiguous() or _dt(p) != x_dt or p.numel() < 1:
                raise ValueError("weight tensors must be contiguous, non-empty and of one dtype")
            n[t] = p.numel()
            xs[t] = p.data_ptr()
            for m in range(M):
                gt = grads[m][t]
                if not gt.is_contiguous() or _dt(gt) != g_dt or gt.numel() != p.numel():
                    raise ValueError(f"gradient of worker {m}, tensor {t}: must be contiguous, {p.numel()} elements, one dtype")
                gs[t * M + m] = gt.data_ptr()
                if momenta is not None:
                    vt = momenta[m][t]
                    if not vt.is_contiguous() or vt.dtype != torch.float32 or vt.numel() != p.numel():
                        raise ValueError(f"momentum of worker {m}, tensor {t}: must be contiguous fp32, {p.numel()} elements")
                    vs[t * M + m] = vt.data_ptr()
        nbytes = lib.ssv_multi_plan_bytes(T, M, ctypes.cast(n, _c_p))
        if nbytes == 0:
            raise ValueError("bad tensor list (sizes out of range)")
        self.host = torch.zeros((nbytes + 7) // 8, dtype=torch.int64)            # 8-byte aligned host bytes
        _check("ssv_multi_plan_fill",
               lib.ssv_multi_plan_fill(self.host.data_ptr(), nbytes, T, M, ctypes.cast(n, _c_p), ctypes.cast(xs, _c_p),
                                       x_dt, ctypes.cast(gs, _c_p), g_dt,
                                       ctypes.cast(vs, _c_p) if vs is not None else None))
        self.device = self.host.to(dev)
        self.T, self.M, self.numel, self.nbytes, self.dev = T, M, sum(int(k) for k in n), int(nbytes), dev
        self.has_momentum = momenta is not None
        self._keep = (list(params), [list(r) for r in grads], None if momenta is None else [list(r) for r in momenta])


def multi_workspace(plan):
    """A new device buffer of the size ssv_signum_step_multi_ws needs for this plan (the workers' packed signs)."""
    nbytes = load_library().ssv_multi_workspace_bytes(plan.host.data_ptr())
    if nbytes == 0:
        raise ValueError("not a filled plan")
    return torch.empty((nbytes // 8,), dtype=torch.int64, device=plan.dev)


def signum_step_multi(plan, beta, lr, weight_decay=0.0, workspace=None):
    """One iteration of Algorithm 1 over all tensors of the plan: one launch, or -- with a workspace from
    multi_workspace(plan) -- the faster two-kernel form (pack row by row, then vote + update)."""
    lib = load_library()
    if workspace is None:
        _check("ssv_signum_step_multi",
               lib.ssv_signum_step_multi(plan.host.data_ptr(), plan.device.data_ptr(), float(beta), float(lr),
                                         float(weight_decay), _stream(plan.dev)))
        return
    if workspace.dtype != torch.int64 or not workspace.is_contiguous() or workspace.device != plan.device.device:
        raise ValueError("workspace must be a contiguous int64 tensor on the plan's device")
    _check("ssv_signum_step_multi_ws",
           lib.ssv_signum_step_multi_ws(plan.host.data_ptr(), plan.device.data_ptr(), workspace.data_ptr(),
                                        workspace.numel() * 8, float(beta), float(lr), float(weight_decay),
                                        _stream(plan.dev)))


# ---- ternary QSGD (include/signvote_qsgd.h) ----------------------------------------------------------------

def _norms_vec(norms, M):
    if norms.dtype != torch.float32 or _vec(norms).numel() != M:
        raise ValueError(f"norms must be {M} contiguous fp32 values")
    return norms


def qsgd_workspace(M, device):
    """Scratch space for qsgd_norms (per-workgroup partial results), as a float64 tensor."""
    nbytes = load_library().ssv_qsgd_workspace_bytes(int(M))
    if nbytes == 0:
        raise ValueError("M out of range")
    return torch.empty((nbytes // 8,), dtype=torch.float64, device=device)


def qsgd_norms(g, kind, norms=None, workspace=None):
    """norms[m] = Euclidean norm (SSV_QSGD_L2) or largest magnitude (SSV_QSGD_MAX) of row m of g."""
    M, d, gs = _rows(g)
    if norms is not None:
        _norms_vec(norms, M)
    dev = _dev(g, norms, workspace)
    if norms is None:
        norms = torch.empty((M,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = qsgd_workspace(M, dev)
    if not workspace.is_contiguous():
        raise ValueError("workspace must be contiguous")
    _check("ssv_qsgd_norms",
           load_library().ssv_qsgd_norms(_ptr(g), _dt(g), M, d, gs, int(kind), _ptr(norms), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(dev)))
    return norms


def qsgd_norms_static(g, kind, norms):
    """qsgd_norms with the library's built-in scratch space (M <= 256): allocates nothing, so `norms` is required."""
    M, d, gs = _rows(g)
    _norms_vec(norms, M)
    dev = _dev(g, norms)
    _check("ssv_qsgd_norms_static",
           load_library().ssv_qsgd_norms_static(_ptr(g), _dt(g), M, d, gs, int(kind), _ptr(norms), _stream(dev)))
    return norms


def qsgd_quantize(g, u, norms, nonzero=None, sign=None):
    """Packed (nonzero, sign) planes of the ternary quantiser: keep coordinate i of row m iff u * norms[m] < |g|."""
    M, d, gs = _rows(g)
    Mu, du, us = _rows(u)
    if (Mu, du) != (M, d) or u.dtype != torch.float32:
        raise ValueError("u must be fp32 with the shape of g")
    _norms_vec(norms, M)
    ss = None
    if (nonzero is None) != (sign is None):
        raise ValueError("give both planes or neither")
    if nonzero is not None:
        ss = _packed_rows(nonzero, M, d, "nonzero")
        if _packed_rows(sign, M, d, "sign") != ss:
            raise ValueError("the two planes must have the same row stride")
    dev = _dev(g, u, norms, nonzero, sign)
    if nonzero is None:
        nonzero = torch.empty((M, words_for(d)), dtype=torch.int64, device=dev)
        sign = torch.empty((M, words_for(d)), dtype=torch.int64, device=dev)
        ss = words_for(d)
    _check("ssv_qsgd_quantize",
           load_library().ssv_qsgd_quantize(_ptr(g), _dt(g), _ptr(u), _ptr(norms), M, d, gs, us, _ptr(nonzero),
                                            _ptr(sign), ss, _stream(dev)))
    return nonzero, sign


def qsgd_aggregate_apply(nonzero, sign, norms, d, avg_out=None, x=None, lr=0.0):
    """a = average over the workers of norms[m] * q_m; avg_out <- a and / or x <- x - lr a."""
    d = _dim(d)
    M = nonzero.shape[0] if nonzero.dim() == 2 else 0
    ss = _packed_rows(nonzero, M, d, "nonzero")
    if _packed_rows(sign, M, d, "sign") != ss:
        raise ValueError("the two planes must have the same row stride")
    _norms_vec(norms, M)
    if avg_out is None and x is None:
        raise ValueError("give avg_out, x or both")
    if avg_out is not None and (avg_out.dtype != torch.float32 or _vec(avg_out).numel() != d):
        raise ValueError(f"avg_out must be {d} contiguous fp32 values")
    if x is not None:
        _weights(x, d)
    dev = _dev(nonzero, sign, norms, avg_out, x)
    _check("ssv_qsgd_aggregate_apply",
           load_library().ssv_qsgd_aggregate_apply(_ptr(nonzero), _ptr(sign), _ptr(norms), M, d, ss, _ptr(avg_out),
                                                   _ptr(x), _dt(x) if x is not None else SSV_F32, float(lr), _stream(dev)))
    return avg_out if avg_out is not None else x


def bench_copy(src, dst):
    """dst <- src with the library's plain streaming copy kernel (bandwidth yardstick, counter calibration)."""
    dev = _dev(src, dst)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not src.is_contiguous() or not dst.is_contiguous():
        raise ValueError("src and dst must be contiguous and of equal size")
    _check("ssv_bench_copy", load_library().ssv_bench_copy(_ptr(src), _ptr(dst), nbytes, _stream(dev)))
    return dst
