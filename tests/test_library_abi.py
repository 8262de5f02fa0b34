"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments before touching the GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

import paper_2405_01943_amd as dass
from paper_2405_01943_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return dass.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "dass.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dass_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert dass.version() >= 100
    names = [lib.dass_status_string(i).decode() for i in range(8)]
    assert names[0] == "DASS_OK" and len(set(names)) == 8
    assert lib.dass_status_string(99) == b"DASS_ERR_UNKNOWN"


def test_workspace_queries(lib):
    assert lib.dass_calib_workspace_bytes(262144, 4096, 11008, 1) == 0
    assert lib.dass_nm_workspace_bytes(11008, 4096, 0) >= 4 * 11008
    assert lib.dass_nm_workspace_bytes(4096, 11008, 1) >= 4 * 11008
    assert lib.dass_unstructured_workspace_bytes(4096, 14336, 1, 1, 1) >= 4 * 14336
    # column lines of a large matrix: the counts and lists of the passes over 64-column tiles
    # (16-bit counts of 258 slots per column and row slab, 256 list entries of 16 bytes per column)
    tiled = lib.dass_unstructured_workspace_bytes(11008, 4096, 1, 0, 0)
    assert tiled >= 4 * 11008 + 4096 * (4 * 258 * 2 + 256 * 16)   # 4 row slabs for this shape
    assert tiled < 64 << 20
    # a factor that does not vary along the column lines takes other kernels: the factor vector and little more
    assert lib.dass_unstructured_workspace_bytes(11008, 4096, 1, 1, 0) < 1 << 20
    # row lines: the factor vector, the flag block, one word per block of rows
    rows = lib.dass_unstructured_workspace_bytes(4096, 11008, 1, 1, 1)
    assert 4 * 11008 + 4096 // 8 * 4 <= rows < 1 << 20
    # a small matrix: the factor vector and the flag block
    assert lib.dass_unstructured_workspace_bytes(64, 64, 1, 0, 0) <= 1024
    # column lines too long for one workgroup's registers, factor across them: the transposed copy
    assert lib.dass_unstructured_workspace_bytes(24576, 3072, 1, 1, 0) >= 24576 * 3072 * 2


FAKE = ctypes.c_void_p(0x1000)      # aligned, never dereferenced: every call below is rejected first
ODD = ctypes.c_void_p(0x1004)
FAKE2 = ctypes.c_void_p(0x10000000)  # aligned, far from FAKE
FAKE3 = ctypes.c_void_p(0x20000000)


def _nm(lib, W=FAKE, rows=64, cols=64, ld=64, dt=1, norms=FAKE, na=1, ga=1, alpha=1.0, n=2, m=4,
        ws=FAKE, wsb=4096):
    return lib.dass_status_string(lib.dass_score_mask_nm(W, rows, cols, ld, dt, norms, na, ga, alpha,
                                                         n, m, None, ws, wsb, None)).decode()


def test_nm_rejections(lib):
    assert _nm(lib, W=None) == "DASS_ERR_NULL"
    assert _nm(lib, norms=None) == "DASS_ERR_NULL"
    assert _nm(lib, dt=5) == "DASS_ERR_DTYPE"
    assert _nm(lib, rows=0) == "DASS_ERR_SHAPE"
    assert _nm(lib, ld=56) == "DASS_ERR_SHAPE"
    assert _nm(lib, cols=60, ld=64) == "DASS_ERR_SHAPE"          # cols % 8
    assert _nm(lib, rows=6, na=0, ga=0) == "DASS_ERR_SHAPE"      # 6 rows, groups of 4
    assert _nm(lib, m=3) == "DASS_ERR_ARG"
    assert _nm(lib, n=4, m=4) == "DASS_ERR_ARG"
    assert _nm(lib, n=0) == "DASS_ERR_ARG"
    assert _nm(lib, alpha=-0.5) == "DASS_ERR_ARG"
    assert _nm(lib, alpha=float("nan")) == "DASS_ERR_ARG"
    assert _nm(lib, na=2) == "DASS_ERR_ARG"
    assert _nm(lib, W=ODD) == "DASS_ERR_ALIGN"
    assert _nm(lib, ld=68) == "DASS_ERR_ALIGN"                   # bf16 stride % 8
    assert _nm(lib, ws=None) == "DASS_ERR_WORKSPACE"
    assert _nm(lib, wsb=8) == "DASS_ERR_WORKSPACE"
    assert "workspace" in lib.dass_last_error_string().decode()


def test_unstructured_rejections(lib):
    def call(n_prune=8, cols=64, ws=FAKE, wsb=4096, W=FAKE):
        rc = lib.dass_score_mask_unstructured(W, 64, cols, 64, 1, FAKE, 1, 1, 1.0, n_prune, None,
                                              ws, wsb, None)
        return lib.dass_status_string(rc).decode()
    assert call(n_prune=-1) == "DASS_ERR_ARG"
    assert call(n_prune=65) == "DASS_ERR_ARG"
    assert call(ws=None) == "DASS_ERR_WORKSPACE"
    assert call(W=None) == "DASS_ERR_NULL"
    assert call(cols=12) == "DASS_ERR_SHAPE"


def test_unstructured_static_size_limit_precedes_any_gpu_call(lib):
    """More norms than the library's own scratch holds: rejected on the host, with the limit in the text."""
    rc = lib.dass_score_mask_unstructured_static(FAKE, 65544, 8, 8, 1, FAKE, 0, 1, 1.0, 4, None, None)
    assert lib.dass_status_string(rc) == b"DASS_ERR_WORKSPACE"
    assert "65536" in lib.dass_last_error_string().decode()


def test_calib_too_many_tiles_is_rejected_before_the_first_launch(lib):
    # 2^31 tiles of 256 tokens: no launch can hold them; sumsq (a fake pointer) is never written
    rc = lib.dass_calib_norms(FAKE, 1 << 40, 64, FAKE, FAKE, 64, 64, 128, 1, 0, FAKE, 0, None, None, 0, None)
    assert lib.dass_status_string(rc) == b"DASS_ERR_SHAPE"


def test_calib_rejections(lib):
    def call(X=FAKE, T=16, ldx=64, d=64, d_int=8, dt=1, act=0, sumsq=FAKE, ldw=64):
        rc = lib.dass_calib_norms(X, T, ldx, FAKE, FAKE, ldw, d, d_int, dt, act, sumsq, 0, None,
                                  None, 0, None)
        return lib.dass_status_string(rc).decode()
    assert call(X=None) == "DASS_ERR_NULL"
    assert call(sumsq=None) == "DASS_ERR_NULL"
    assert call(dt=2) == "DASS_ERR_DTYPE"
    assert call(act=4) == "DASS_ERR_DTYPE"
    assert call(T=0) == "DASS_ERR_SHAPE"
    assert call(d=60, ldx=64) == "DASS_ERR_SHAPE"                # bf16 needs d % 8
    assert call(ldx=32) == "DASS_ERR_SHAPE"
    assert call(X=ODD) == "DASS_ERR_ALIGN"
    assert call(ldw=68) == "DASS_ERR_ALIGN"


def _task(W=FAKE, rows=64, cols=64, ld=64, norms=FAKE, na=1, ga=1, alpha=1.0, mask=None):
    return binding.NmTask(W.value if W else None, rows, cols, ld, norms.value if norms else None, na, ga, alpha, mask)


def _batched(lib, tasks, dt=1, n=2, m=4, ws=FAKE, wsb=4096):
    arr = (binding.NmTask * max(len(tasks), 1))(*tasks)
    st = lib.dass_score_mask_nm_batched(arr, len(tasks), dt, n, m, ws, wsb, None)
    return lib.dass_status_string(st).decode(), lib.dass_last_error_string().decode()


def test_batched_rejections_name_the_task(lib):
    """Every task is checked before anything is launched; the message carries the offender's index."""
    good = _task()
    assert _batched(lib, [])[0] == "DASS_OK"                       # nothing to do
    name, text = _batched(lib, [good, _task(W=None)])
    assert name == "DASS_ERR_NULL" and "task 1" in text
    name, text = _batched(lib, [good, good, _task(cols=60)])
    assert name == "DASS_ERR_SHAPE" and "task 2" in text
    assert _batched(lib, [good], m=3)[0] == "DASS_ERR_ARG"
    assert _batched(lib, [good], n=4, m=4)[0] == "DASS_ERR_ARG"
    assert _batched(lib, [_task(W=ODD)])[0] == "DASS_ERR_ALIGN"
    assert _batched(lib, [good], wsb=16)[0] == "DASS_ERR_WORKSPACE"
    assert lib.dass_score_mask_nm_batched(None, 3, 1, 2, 4, FAKE, 4096, None) != 0
    arr = (binding.NmTask * 2)(_task(rows=4096, cols=11008, ld=11008), _task(rows=11008, cols=4096, ld=4096, na=0, ga=0))
    assert lib.dass_nm_batched_workspace_bytes(arr, 2) >= 4 * 11008


def _inorm(lib, X=FAKE, T=64, ldx=64, d=64, dt=1, sumsq=FAKE, norms=None, ws=FAKE, wsb=1 << 20):
    return lib.dass_status_string(lib.dass_input_norms(X, T, ldx, d, dt, sumsq, 0, norms, ws, wsb, None)).decode()


def test_input_norms_rejections(lib):
    assert _inorm(lib, X=None) == "DASS_ERR_NULL"
    assert _inorm(lib, sumsq=None) == "DASS_ERR_NULL"
    assert _inorm(lib, dt=7) == "DASS_ERR_DTYPE"
    assert _inorm(lib, T=0) == "DASS_ERR_SHAPE"
    assert _inorm(lib, d=60) == "DASS_ERR_SHAPE"
    assert _inorm(lib, ldx=56) == "DASS_ERR_SHAPE"
    assert _inorm(lib, X=ODD) == "DASS_ERR_ALIGN"
    assert _inorm(lib, norms=ODD) == "DASS_ERR_ALIGN"
    assert _inorm(lib, ldx=68, dt=1) == "DASS_ERR_ALIGN"        # bf16 rows must start on 16 bytes
    assert _inorm(lib, ws=None) == "DASS_ERR_WORKSPACE"
    assert _inorm(lib, wsb=64) == "DASS_ERR_WORKSPACE"
    assert lib.dass_input_norms_workspace_bytes(262144, 4096) >= 512 * 4096 * 4
    assert lib.dass_input_norms_workspace_bytes(0, 4096) == 0


def _fwd(lib, X=FAKE, T=256, ldx=128, Wg=FAKE, Wu=FAKE, ldw=128, Wd=FAKE, ldd=192, d=128, d_int=192, dt=1, act=0,
         out=FAKE, ldo=128, ws=FAKE, wsb=1 << 20):
    return lib.dass_status_string(lib.dass_mlp_forward(X, T, ldx, Wg, Wu, ldw, Wd, ldd, d, d_int, dt, act, out, ldo,
                                                       ws, wsb, None)).decode()


def test_mlp_forward_rejections(lib):
    assert _fwd(lib, X=None) == "DASS_ERR_NULL"
    assert _fwd(lib, out=None) == "DASS_ERR_NULL"               # out may be absent only together with Wdown
    assert _fwd(lib, Wd=None, out=None, ldd=0, ldo=0, wsb=64) == "DASS_ERR_WORKSPACE"   # Eq. 2 alone: still checked
    assert _fwd(lib, ws=None) == "DASS_ERR_NULL"
    assert _fwd(lib, dt=0) == "DASS_ERR_DTYPE"                  # bf16 only
    assert _fwd(lib, act=9) == "DASS_ERR_DTYPE"
    assert _fwd(lib, T=0) == "DASS_ERR_SHAPE"
    assert _fwd(lib, d=96, ldx=96, ldw=96, ldo=96) == "DASS_ERR_SHAPE"     # multiples of 64
    assert _fwd(lib, d_int=200, ldd=200) == "DASS_ERR_SHAPE"
    assert _fwd(lib, ldd=128) == "DASS_ERR_SHAPE"
    assert _fwd(lib, out=ODD) == "DASS_ERR_ALIGN"
    assert _fwd(lib, ldo=132) == "DASS_ERR_ALIGN"
    assert _fwd(lib, wsb=256 * 192 * 2 - 1) == "DASS_ERR_WORKSPACE"
    assert lib.dass_mlp_forward_workspace_bytes(256, 128, 192, 1) == 256 * 192 * 2
    assert lib.dass_mlp_forward_workspace_bytes(256, 128, 192, 0) == 0


def _cmp(lib, W=FAKE, rows=64, cols=64, ld=64, dt=1, axis=1, V=FAKE2, ldv=32, M=FAKE3, ldm=8, surplus=None):
    return lib.dass_status_string(lib.dass_compress_24(W, rows, cols, ld, dt, axis, V, ldv, M, ldm, surplus,
                                                       None)).decode()


def test_compress_rejections(lib):
    assert _cmp(lib, W=None) == "DASS_ERR_NULL"
    assert _cmp(lib, M=None) == "DASS_ERR_NULL"
    assert _cmp(lib, dt=5) == "DASS_ERR_DTYPE"
    assert _cmp(lib, axis=2) == "DASS_ERR_ARG"
    assert _cmp(lib, cols=60, ld=64) == "DASS_ERR_SHAPE"                       # cols % 8
    assert _cmp(lib, axis=0, rows=62, ldv=64, ldm=32) == "DASS_ERR_SHAPE"      # rows % 4
    assert _cmp(lib, ldv=24) == "DASS_ERR_SHAPE"
    assert _cmp(lib, ldm=4) == "DASS_ERR_SHAPE"
    assert _cmp(lib, V=ODD) == "DASS_ERR_ALIGN"
    assert _cmp(lib, axis=0, ldv=64, ldm=34) == "DASS_ERR_ALIGN"              # codes are written 4 bytes at a time
    assert _cmp(lib, ldv=34) == "DASS_ERR_ALIGN"
    assert _cmp(lib, surplus=ODD) == "DASS_ERR_ALIGN"
    assert _cmp(lib, V=FAKE) == "DASS_ERR_ARG"                                 # values_out on top of W


def _spd(lib, Y=FAKE, T=256, ldy=192, V=FAKE2, ldv=96, M=FAKE3, ldm=24, d=128, d_int=192, dt=1, out=FAKE, ldo=128):
    return lib.dass_status_string(lib.dass_down_proj_sparse24(Y, T, ldy, V, ldv, M, ldm, d, d_int, dt, out, ldo,
                                                              None)).decode()


def test_sparse_down_rejections(lib):
    assert _spd(lib, Y=None) == "DASS_ERR_NULL"
    assert _spd(lib, M=None) == "DASS_ERR_NULL"
    assert _spd(lib, dt=0) == "DASS_ERR_DTYPE"
    assert _spd(lib, T=0) == "DASS_ERR_SHAPE"
    assert _spd(lib, d_int=200, ldy=200, ldv=104, ldm=28) == "DASS_ERR_SHAPE"   # d_int % 64
    assert _spd(lib, d=100) == "DASS_ERR_SHAPE"                                # d % 8
    assert _spd(lib, ldv=88) == "DASS_ERR_SHAPE"
    assert _spd(lib, ldm=20) == "DASS_ERR_SHAPE"
    assert _spd(lib, V=ODD) == "DASS_ERR_ALIGN"
    assert _spd(lib, ldm=26) == "DASS_ERR_ALIGN"
    assert _spd(lib, ldo=132) == "DASS_ERR_ALIGN"
