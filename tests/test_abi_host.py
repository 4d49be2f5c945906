"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares, and
rejects bad arguments before anything is launched (no GPU needed: validation never dereferences)."""
import ctypes
import os
import re

import pytest

import paper_2412_07174_amd as scap
from paper_2412_07174_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000   # 16-byte aligned, never dereferenced: every call below fails validation first
ODD = FAKE + 2


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(scap.lib_path()):
        from paper_2412_07174_amd import build
        build.build(verbose=False)
    return scap.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "scap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(scap_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings_and_version(lib):
    assert scap.version() >= 100
    assert scap.status_string(0) == "ok"
    seen = {scap.status_string(c) for c in range(-9, 1)}
    assert len(seen) == 10 and "unknown status" not in seen
    assert scap.status_string(-99) == "unknown status"


def test_workspace_bytes(lib):
    assert scap.workspace_bytes(14336, 4096, 1) >= 4 * (1 << 20)
    assert 0 < scap.workspace_bytes(1024, 0, 256) < scap.workspace_bytes(1024, 8, 1)   # calibration-only
    assert scap.workspace_bytes(0, 4096, 1) == 0
    assert scap.workspace_bytes(4096, 4096, 17) == 0
    assert scap.workspace_bytes(4096, 4096, 16) > scap.workspace_bytes(4096, 4096, 1)


def _fc(lib, **kw):
    a = dict(W=FAKE, col_scale=None, K=1024, N=4096, wdt=1, x=FAKE, xdt=1, B=1, m=0.0, tau=0.5, b=None, y=FAKE,
             idx=None, nnz=None, unz=None, ws=FAKE, wsb=1 << 30, stream=None)
    a.update(kw)
    return lib.scap_sparse_fc(a["W"], a["col_scale"], a["K"], a["N"], a["wdt"], a["x"], a["xdt"], a["B"], a["m"],
                              a["tau"], a["b"], a["y"], a["idx"], a["nnz"], a["unz"], a["ws"], a["wsb"], a["stream"])


def test_sparse_fc_argument_validation(lib):
    assert _fc(lib, W=None) == -1
    assert _fc(lib, x=None) == -1
    assert _fc(lib, y=None) == -1
    assert _fc(lib, wdt=2) == -1                      # int8 without column scales
    assert _fc(lib, idx=FAKE) == -1                   # idx_out needs nnz_out
    assert _fc(lib, N=4100) == -2                     # not a multiple of 8
    assert _fc(lib, wdt=2, col_scale=FAKE, N=4104) == -2   # int8 wants multiples of 16
    assert _fc(lib, K=0) == -2
    assert _fc(lib, B=0) == -2 and _fc(lib, B=17) == -2
    assert _fc(lib, wdt=7) == -3 and _fc(lib, xdt=2) == -3
    assert _fc(lib, W=ODD) == -4 and _fc(lib, x=ODD) == -4 and _fc(lib, y=ODD) == -4 and _fc(lib, b=ODD) == -4
    assert _fc(lib, tau=-0.1) == -5
    assert _fc(lib, tau=float("nan")) == -5 and _fc(lib, tau=float("inf")) == -5
    assert _fc(lib, m=float("inf")) == -5
    assert _fc(lib, ws=None) == -6
    assert _fc(lib, wsb=1000) == -6
    assert _fc(lib, ws=ODD) == -4


def test_other_entry_points_validate(lib):
    f = ctypes.c_float(0)
    p = ctypes.byref(f)
    assert lib.scap_calibrate(None, 4, 8, 1, 0.5, 2, p, p, FAKE, 1 << 21, None) == -1
    assert lib.scap_calibrate(FAKE, 4, 8, 1, 0.5, 2, None, p, FAKE, 1 << 21, None) == -1
    assert lib.scap_calibrate(FAKE, 4, 8, 2, 0.5, 2, p, p, FAKE, 1 << 21, None) == -3
    assert lib.scap_calibrate(FAKE, 4, 8, 1, 0.5, 9, p, p, FAKE, 1 << 21, None) == -3
    assert lib.scap_calibrate(FAKE, 0, 8, 1, 0.5, 2, p, p, FAKE, 1 << 21, None) == -2
    assert lib.scap_calibrate(FAKE, 4, 8, 1, 1.0, 2, p, p, FAKE, 1 << 21, None) == -5
    assert lib.scap_calibrate(FAKE, 4, 8, 1, -0.1, 2, p, p, FAKE, 1 << 21, None) == -5
    assert lib.scap_calibrate(FAKE, 4, 8, 1, 0.5, 2, p, p, FAKE, 100, None) == -6
    assert lib.scap_fold_bias(None, None, 8, 8, 1, None, 0.0, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.scap_fold_bias(FAKE, None, 8, 8, 1, None, float("nan"), FAKE, FAKE, 1 << 30, None) == -5
    assert lib.scap_fold_bias(FAKE, None, 8, 12, 1, None, 0.0, FAKE, FAKE, 1 << 30, None) == -2
    assert lib.scap_dense_fc(FAKE, None, 8, 8, 1, None, 1, 1, None, FAKE, FAKE, 1 << 30, None, None) == -1
    assert lib.scap_workspace_init(None, 1 << 20, None) == -6
    assert lib.scap_workspace_init(FAKE, 16, None) == -6
    assert lib.scap_read_probe(None, 1024, FAKE, None) == -1
    assert lib.scap_read_probe(FAKE, 1000, FAKE, None) == -2


def _blk(lib, **kw):
    a = dict(Wgu=FAKE, sgu=None, Wd=FAKE, sd=None, K=4096, F=14336, N=4096, wdt=1, x=FAKE, xdt=1, B=1, mx=0.0, tx=0.5,
             bgu=None, mz=0.0, tz=0.1, bd=None, y=FAKE, z=None, idx=None, nnz=None, ws=FAKE, wsb=1 << 30, stream=None)
    a.update(kw)
    return lib.scap_swiglu_block(a["Wgu"], a["sgu"], a["Wd"], a["sd"], a["K"], a["F"], a["N"], a["wdt"], a["x"], a["xdt"],
                                 a["B"], a["mx"], a["tx"], a["bgu"], a["mz"], a["tz"], a["bd"], a["y"], a["z"], a["idx"],
                                 a["nnz"], a["ws"], a["wsb"], a["stream"])


def test_swiglu_block_entry_points_validate(lib):
    assert scap.swiglu_workspace_bytes(4096, 14336, 4096, 1) >= max(scap.workspace_bytes(4096, 28672, 1),
                                                                    scap.workspace_bytes(14336, 4096, 1))
    assert scap.swiglu_workspace_bytes(4096, 0, 4096, 1) == 0
    assert scap.swiglu_workspace_bytes(4096, 1 << 19, 4096, 1) == 0
    assert _blk(lib, Wgu=None) == -1
    assert _blk(lib, Wd=None) == -1
    assert _blk(lib, x=None) == -1
    assert _blk(lib, y=None) == -1
    assert _blk(lib, idx=FAKE) == -1                 # list without a count
    assert _blk(lib, F=14338) == -2                  # not a multiple of 4
    assert _blk(lib, F=0) == -2
    assert _blk(lib, N=4100) == -2
    assert _blk(lib, wdt=2) == -1                    # int8 without scales
    assert _blk(lib, wdt=2, sgu=FAKE, sd=FAKE, F=14340) == -2   # int8: 2F must be a multiple of 16
    assert _blk(lib, wdt=7) == -3
    assert _blk(lib, xdt=2) == -3
    assert _blk(lib, B=0) == -2
    assert _blk(lib, B=17) == -2
    assert _blk(lib, x=ODD) == -4
    assert _blk(lib, z=ODD) == -4
    assert _blk(lib, tx=-0.5) == -5
    assert _blk(lib, tz=float("inf")) == -5
    assert _blk(lib, mz=float("nan")) == -5
    assert _blk(lib, ws=None) == -6
    assert _blk(lib, wsb=1 << 20) == -6
    assert lib.scap_pack_gate_up(None, FAKE, 4, 8, 2, FAKE, None) == -1
    assert lib.scap_pack_gate_up(FAKE, FAKE, 4, 8, 3, FAKE, None) == -3
    assert lib.scap_pack_gate_up(FAKE, FAKE, 4, 6, 2, FAKE, None) == -2
    assert lib.scap_pack_gate_up(FAKE, FAKE, 0, 8, 2, FAKE, None) == -2
    assert lib.scap_pack_gate_up(FAKE, ODD, 4, 8, 2, FAKE, None) == -4


def test_product_package_does_not_touch_the_oracle():
    """The product path must not import, link or call the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2412_07174_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "scap_oracle" not in text, f


def test_binding_refuses_tensors_the_kernels_would_overrun(lib):
    """The binding hands raw pointers to the kernels, so it checks dtype, layout, shape and device of every tensor
    first (CPU tensors suffice here: the device check comes last and nothing is launched)."""
    import torch

    class FakeWs:
        pass

    K, N = 64, 32
    W = torch.zeros((K, N), dtype=torch.bfloat16)
    x = torch.zeros(K, dtype=torch.bfloat16)
    ws = FakeWs()
    with pytest.raises(ValueError, match="contiguous"):        # a torch Linear weight viewed as [K, N]
        scap.sparse_fc(torch.zeros((N, K), dtype=torch.bfloat16).t(), x, 0.0, 0.1, workspace=ws)
    with pytest.raises(ValueError, match="shape"):             # input shorter than K
        scap.sparse_fc(W, x[:-8], 0.0, 0.1, workspace=ws)
    with pytest.raises(TypeError, match="dtype"):
        scap.sparse_fc(W, x.float(), 0.0, 0.1, workspace=ws)
    with pytest.raises(TypeError, match="dtype"):
        scap.sparse_fc(W.float(), x, 0.0, 0.1, workspace=ws)
    with pytest.raises(TypeError, match="required"):           # int8 weights without their scales
        scap.sparse_fc(W.to(torch.int8), x, 0.0, 0.1, workspace=ws)
    with pytest.raises(ValueError, match="shape"):             # undersized output
        scap.sparse_fc(W, x, 0.0, 0.1, y=torch.zeros((1, N - 8)), workspace=ws)
    with pytest.raises(ValueError, match="shape"):             # undersized index list
        scap.sparse_fc(W, x, 0.0, 0.1, idx_out=torch.zeros((1, K - 1), dtype=torch.int32),
                       nnz_out=torch.zeros(1, dtype=torch.int32), workspace=ws)
    with pytest.raises(ValueError, match="shape"):
        scap.sparse_fc(W, x, 0.0, 0.1, torch.zeros(N + 8), workspace=ws)
    with pytest.raises(ValueError, match="shape"):
        scap.dense_fc(W, torch.zeros((3, K + 1), dtype=torch.bfloat16), workspace=ws)
    with pytest.raises(ValueError, match="shape"):
        scap.fold_bias(W, 0.1, torch.zeros(N - 1), workspace=ws)
    with pytest.raises(ValueError, match="expected"):
        scap.calibrate(x, 0.5, workspace=ws)                    # a vector, not [n, K]
    with pytest.raises(ValueError, match="W_down has"):
        scap.swiglu_block(W, torch.zeros((N, 8), dtype=torch.bfloat16), x, 0.0, 0.1, None, 0.0, 0.1, None, workspace=ws)
    with pytest.raises(ValueError, match="GPU"):               # everything right except where it lives
        scap.sparse_fc(W, x, 0.0, 0.1, workspace=ws)
