"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the public
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "signvote.h"), os.path.join(ROOT, "include", "signvote_bench.h")]


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
            "ssv_vote_apply", "ssv_signum_step", "ssv_status_string", "ssv_version", "ssv_bench_copy"} <= set(names)
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


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_1810_05291_amd as sv
    with pytest.raises(ValueError):
        sv.sign_pack(torch.zeros(2, 64))


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
