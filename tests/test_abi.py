"""Host-side checks that need no GPU: the library loads, exports every symbol include/mp.h declares, the ctypes
mirror of the structs has the C layout, and argument validation rejects bad calls before anything is enqueued."""
import ctypes as C
import os
import re
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mp.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mp_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    from paper_1805_10387_amd import _lib
    lib = _lib.load()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mp.h but not exported"
        assert n in _lib.SIGNATURES, f"{n} has no ctypes signature"
    assert set(_lib.SIGNATURES) == set(names)


def test_binding_has_the_same_names():
    import paper_1805_10387_amd as mp
    for n in _declared():
        if n == "mp_last_error":
            continue
        assert hasattr(mp, n), f"binding lacks {n}"


def test_struct_layouts_match_the_header():
    from paper_1805_10387_amd import _lib
    assert C.sizeof(_lib.ScaleState) == 12 * 4 + _lib.MP_HISTORY * 8
    assert _lib.ScaleState.found_inf.offset == 28 and _lib.ScaleState.opt_step.offset == 32
    assert _lib.ScaleState.hist_scale.offset == 48
    assert C.sizeof(_lib.GemmDesc) == 8 * 4 + 6 * 8 + 4 * 4
    assert _lib.GemmDesc.sx_outer.offset == 32 and _lib.GemmDesc.alpha.offset == 80
    assert C.sizeof(_lib.TensorDesc) == 48 and C.sizeof(_lib.OptCfg) == 48
    hdr = open(HEADER).read()
    assert f"#define MP_HISTORY {_lib.MP_HISTORY}" in hdr


def test_validation_errors_enqueue_nothing():
    """NULL / malformed arguments are rejected on the host (no HIP call is made on these paths)."""
    from paper_1805_10387_amd import _lib
    lib = _lib.load()
    assert lib.mp_version() >= 1
    assert lib.mp_scale_state_init(None, 1, 2.0, 1, 1.0, 4.0, None) == _lib.MP_E_INVAL
    assert b"NULL" in lib.mp_last_error()
    assert lib.mp_loss_scale_update(None, None) == _lib.MP_E_INVAL
    d = _lib.GemmDesc()
    d.M, d.N, d.K, d.ldx, d.ldw, d.ldy, d.batch_outer, d.batch_inner, d.alpha = 8, 8, 8, 8, 8, 8, 1, 1, 1.0
    assert lib.mp_gemm_fwd(C.byref(d), None, None, None, None, None, None, None) == _lib.MP_E_INVAL
    d.ldx = 4
    assert lib.mp_gemm_bwd_dx(C.byref(d), 16, 16, None, None, 0, 16, None) == _lib.MP_E_INVAL
    assert b"leading dimension" in lib.mp_last_error()
    d.ldx = 8
    assert lib.mp_gemm_bwd_dw(C.byref(d), 16, 16, 16, None, None, None, 0, None) == _lib.MP_E_WORKSPACE
    cfg = _lib.OptCfg()
    cfg.kind = 7
    assert lib.mp_unscale_check_update(None, 0, C.byref(cfg), 16, 0, None) == _lib.MP_E_INVAL
    assert lib.mp_layernorm_fwd(4, 12, 16, None, 16, 16, 1e-5, 16, 16, 16, None) == _lib.MP_E_UNSUPPORTED
    assert lib.mp_mse_scaled(4, 8, 16, 16, 4, 16, 16, 16, None, 0, None) == _lib.MP_E_INVAL      # ld < cols
    # cross-entropy with the bias gradient: shape, NULL and workspace errors come before any launch
    assert lib.mp_softmax_xent_scaled_db(4, 8, 16, 4, 16, 16, 16, 16, 16, 16, 1 << 20, None) == _lib.MP_E_INVAL   # ld < vocab
    assert lib.mp_softmax_xent_scaled_db(4, 8, 16, 8, 16, 16, 16, 16, None, 16, 1 << 20, None) == _lib.MP_E_INVAL  # db NULL
    assert lib.mp_softmax_xent_scaled_db(4, 8, 16, 8, 16, 16, 16, 16, 16, 16, 8, None) == _lib.MP_E_WORKSPACE
    assert lib.mp_softmax_xent_db_workspace_bytes(0, 8) == 0
    assert lib.mp_softmax_xent_db_workspace_bytes(8192, 32768) >= 256 * 32768 * 4 + 8192 * 4
    assert C.sizeof(_lib.GemmGroupItem) == C.sizeof(_lib.GemmDesc) + 4 * 8
    # grouped weight gradients: empty / oversized lists, and shapes the grouped kernel does not take
    assert lib.mp_gemm_bwd_dw_grouped(None, 0, None, None) == _lib.MP_E_INVAL
    items = (_lib.GemmGroupItem * 9)()
    assert lib.mp_gemm_bwd_dw_grouped(items, 9, None, None) == _lib.MP_E_INVAL
    it = items[0]
    it.desc.M, it.desc.N, it.desc.K, it.desc.ldx, it.desc.ldw, it.desc.ldy = 128, 136, 128, 128, 128, 136
    it.desc.batch_outer = it.desc.batch_inner = 1
    it.desc.alpha = 1.0
    it.dY = it.X = it.dW = 256
    assert lib.mp_gemm_bwd_dw_grouped(items, 1, None, None) == _lib.MP_E_UNSUPPORTED     # 136 is not a multiple of 128
    assert b"mp_gemm_bwd_dw" in lib.mp_last_error()
    it.desc.N, it.desc.ldy, it.dW = 128, 128, None
    assert lib.mp_gemm_bwd_dw_grouped(items, 1, None, None) == _lib.MP_E_INVAL            # NULL operand
    # matrix-core rate probe: buffers are checked before anything is launched
    out = C.c_double(0.0)
    assert lib.mp_mfma_sustained_rate(None, 0, None, 0, 1, 1, C.byref(out), None) == _lib.MP_E_INVAL
    assert lib.mp_mfma_sustained_rate(256, 100, 256, 1 << 20, 256, 10, C.byref(out), None) == _lib.MP_E_INVAL   # too few operands
    assert lib.mp_mfma_sustained_rate(256, 16384, 256, 10, 256, 10, C.byref(out), None) == _lib.MP_E_INVAL      # sink too small
    assert lib.mp_mfma_sustained_rate(264, 16384, 256, 1 << 20, 256, 10, C.byref(out), None) == _lib.MP_E_INVAL  # misaligned


def test_workspace_queries_are_consistent():
    from paper_1805_10387_amd import _lib
    lib = _lib.load()
    d = _lib.GemmDesc()
    d.batch_outer = d.batch_inner = 1
    d.alpha = 1.0
    # big output, short contraction: no split, only the column-sum partials
    d.M, d.N, d.K, d.ldx, d.ldw, d.ldy = 8192, 4096, 1024, 1024, 1024, 4096
    no_db, with_db = lib.mp_gemm_bwd_dw_workspace_bytes(C.byref(d), 0), lib.mp_gemm_bwd_dw_workspace_bytes(C.byref(d), 1)
    assert with_db - no_db == lib.mp_colsum_workspace_bytes(8192, 4096) and no_db < (1 << 28)
    # small output, long contraction: split over K -> fp32 partials of (splits x N x K)
    d.M, d.N, d.K, d.ldx, d.ldw, d.ldy = 8192, 128, 256, 256, 256, 128
    split = lib.mp_gemm_bwd_dw_workspace_bytes(C.byref(d), 0)
    assert split >= 2 * 128 * 256 * 4 and (split - 256) % (128 * 256 * 4) == 0
    assert lib.mp_loss_workspace_bytes(8192, 32768) >= 8192 * 4
    assert lib.mp_layernorm_bwd_workspace_bytes(8192, 1024) % (2 * 1024 * 4) == 0


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_1805_10387_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            src = open(os.path.join(pkg, fn)).read()
            assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), fn
    for fn in os.listdir(os.path.join(ROOT, "oracle")):
        if fn.endswith(".py"):
            src = open(os.path.join(ROOT, "oracle", fn)).read()
            assert "paper_1805_10387_amd" not in src, fn


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N with N > 1 exits with a message before touching any device."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
