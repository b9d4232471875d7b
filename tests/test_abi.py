"""The C ABI without a GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before any launch."""
import os
import re

import pytest

from paper_1805_08899_amd import binding as eb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", f) for f in sorted(os.listdir(os.path.join(ROOT, "include")))
           if f.endswith(".h")]


def declared_symbols():
    names = set()
    for h in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(echo_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert "echo_attn_fwd" in names and "echo_attn_bwd" in names and len(names) >= 11
    L = eb.lib()
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(eb.EXPORTS), "binding and header disagree"


def test_version_and_status_strings():
    assert "gfx950" in eb.echo_version()
    seen = {eb.echo_status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen


def test_workspace_queries():
    d = eb.make_desc(64, 50, 50, 512, 512)
    assert eb.echo_attn_fwd_workspace_bytes(d) >= 0
    assert eb.echo_attn_bwd_workspace_bytes(d) >= 64 * 50 * 50 * 4
    assert eb.echo_attn_stash_bytes(d) == 64 * 50 * 50 * 512 * 4
    bad = eb.make_desc(0, 50, 50, 512, 512)
    assert eb.echo_attn_fwd_workspace_bytes(bad) == 0 and eb.echo_attn_bwd_workspace_bytes(bad) == 0
    assert eb.echo_attn_stash_bytes(bad) == 0


A = 0x10000  # a fake, aligned, never dereferenced device address


def _fwd(desc, **kw):
    args = dict(Qp=A, Kp=A, V=A, v=A, key_len=A, context=A, P=A, workspace=A, workspace_bytes=1 << 40)
    args.update(kw)
    return eb.echo_attn_fwd(desc, **args)


def _bwd(desc, **kw):
    args = dict(dContext=A, P=A, Qp=A, Kp=A, V=A, v=A, key_len=A, dQp=A, dKp=A, dV=A, dv=A, workspace=A,
                workspace_bytes=1 << 40)
    args.update(kw)
    return eb.echo_attn_bwd(desc, **args)


def test_rejects_bad_arguments_without_launching():
    good = eb.make_desc(4, 6, 7, 16, 16)
    for name in ("Qp", "Kp", "V", "v", "key_len", "context", "P"):
        assert _fwd(good, **{name: None}) == eb.ECHO_ERR_NULL, name
    # H = 18 is not a multiple of 4: the forward pass keeps its scores in the workspace and must be given one
    unfused = eb.make_desc(4, 6, 7, 18, 16)
    assert eb.echo_attn_fwd_workspace_bytes(unfused) >= 4 * 6 * 7 * 4
    assert _fwd(unfused, workspace=None) == eb.ECHO_ERR_NULL
    assert _fwd(unfused, workspace_bytes=eb.echo_attn_fwd_workspace_bytes(unfused) - 1) == eb.ECHO_ERR_WORKSPACE
    for name in ("dContext", "P", "Qp", "Kp", "V", "v", "key_len", "dQp", "dKp", "dV", "dv", "workspace"):
        assert _bwd(good, **{name: None}) == eb.ECHO_ERR_NULL, name
    assert _fwd(good, Qp=A + 4) == eb.ECHO_ERR_ALIGN
    assert _bwd(good, dKp=A + 8) == eb.ECHO_ERR_ALIGN
    assert _bwd(good, workspace_bytes=eb.echo_attn_bwd_workspace_bytes(good) - 1) == eb.ECHO_ERR_WORKSPACE
    for field in ("B", "Tq", "Tk", "H", "Dv"):
        for val in (0, -3):
            d = eb.make_desc(4, 6, 7, 16, 16)
            setattr(d, field, val)
            assert _fwd(d) == eb.ECHO_ERR_SHAPE and _bwd(d) == eb.ECHO_ERR_SHAPE, (field, val)
    assert _fwd(eb.make_desc(4, 6, 7, 16, 18)) == eb.ECHO_ERR_SHAPE          # Dv not a multiple of 4
    assert _fwd(eb.make_desc(1, 70000, 70, 70000, 16)) == eb.ECHO_ERR_SHAPE  # per-sample tensor >= 2^31 elements
    assert _fwd(eb.make_desc(4, 6, 7, 16, 16, in_dtype=7)) == eb.ECHO_ERR_DTYPE


def test_one_kernel_forward_needs_no_workspace():
    """Shapes that take the one-kernel forward report 0 bytes; the keep-the-map variant still needs the scores."""
    for shape in ((4, 6, 7, 16, 16), (64, 50, 50, 512, 512), (32, 300, 300, 1024, 1024), (2, 9, 64, 2048, 64)):
        d = eb.make_desc(*shape)
        assert eb.echo_attn_fwd_workspace_bytes(d) == 0, shape
        assert eb.echo_attn_fwd_stash_workspace_bytes(d) >= shape[0] * shape[1] * shape[2] * 4, shape
    d = eb.make_desc(4, 6, 7, 16, 16)
    assert eb.echo_attn_fwd_stash(d, A, A, A, A, A, A, A, A, None, 0) == eb.ECHO_ERR_NULL
    assert eb.echo_attn_fwd_stash(d, A, A, A, A, A, A, A, A, A, 16) == eb.ECHO_ERR_WORKSPACE


def test_documented_shape_limits():
    """Each limit of the header's "Shape limits", at the first value past it and (host checks only) at the last one
    inside, through a call that stops at the next check (a NULL tensor) instead of launching."""
    def fwd_rc(*shape):
        return _fwd(eb.make_desc(*shape), Qp=None)

    def bwd_rc(*shape):
        return _bwd(eb.make_desc(*shape), dContext=None)
    assert eb.ECHO_ATTN_MAX_TK == 2048 and eb.ECHO_ATTN_STEP_MAX_TK == 8192 and eb.ECHO_ATTN_MAX_B == 65535
    for rc in (fwd_rc, bwd_rc):
        assert rc(2, 3, eb.ECHO_ATTN_MAX_TK, 8, 8) == eb.ECHO_ERR_NULL
        assert rc(2, 3, eb.ECHO_ATTN_MAX_TK + 1, 8, 8) == eb.ECHO_ERR_SHAPE
        assert rc(eb.ECHO_ATTN_MAX_B, 3, 5, 8, 8) == eb.ECHO_ERR_NULL
        assert rc(eb.ECHO_ATTN_MAX_B + 1, 3, 5, 8, 8) == eb.ECHO_ERR_SHAPE
        for dv in (1, 2, 3, 6, 18):
            assert rc(2, 3, 5, 8, dv) == eb.ECHO_ERR_SHAPE, dv
        assert rc(2, 3, 5, 7, 4) == eb.ECHO_ERR_NULL                   # any H >= 1
    big = eb.make_desc(eb.ECHO_ATTN_MAX_B + 1, 3, 5, 8, 8)
    assert eb.echo_attn_fwd_workspace_bytes(big) == 0 and eb.echo_attn_bwd_workspace_bytes(big) == 0
    assert eb.echo_attn_bwd_static(big, A, A, A, A, A, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    # the step calls take a longer key axis
    step = lambda tk: eb.echo_attn_step_fwd(eb.make_desc(2, 1, tk, 8, 8), None, A, A, A, A, A, A)
    assert step(eb.ECHO_ATTN_MAX_TK + 1) == eb.ECHO_ERR_NULL
    assert step(eb.ECHO_ATTN_STEP_MAX_TK) == eb.ECHO_ERR_NULL
    assert step(eb.ECHO_ATTN_STEP_MAX_TK + 1) == eb.ECHO_ERR_SHAPE
    assert eb.echo_attn_step_finish(eb.make_desc(2, 1, eb.ECHO_ATTN_STEP_MAX_TK + 1, 8, 8), A, A) == eb.ECHO_ERR_SHAPE


def test_null_descriptor():
    import ctypes
    L = eb.lib()
    assert L.echo_attn_fwd(None, A, A, A, A, A, A, A, A, 1 << 40, None) == eb.ECHO_ERR_NULL
    assert L.echo_attn_fwd_workspace_bytes(None) == 0


def test_stash_entry_points_validate_too():
    good = eb.make_desc(4, 6, 7, 16, 16)
    assert eb.echo_attn_fwd_stash(good, A, A, A, A, A, A, A, None, A, 1 << 40) == eb.ECHO_ERR_NULL
    assert eb.echo_attn_bwd_stash(good, A, A, None, A, A, A, A, A, A, A, A, 1 << 40) == eb.ECHO_ERR_NULL


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(eb, "_lib", None)
    monkeypatch.setattr(eb, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        eb.lib()


def test_dropout_rejects_bad_arguments_without_launching():
    assert eb.echo_dropout_mask_words(1) == 1 and eb.echo_dropout_mask_words(32) == 1
    assert eb.echo_dropout_mask_words(33) == 2
    assert eb.echo_dropout_fwd(None, 8, 0.5, 1, 0, A, A) == eb.ECHO_ERR_NULL
    assert eb.echo_dropout_fwd(A, 0, 0.5, 1, 0, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_dropout_fwd(A, (1 << 40) + 1, 0.5, 1, 0, A, A) == eb.ECHO_ERR_SHAPE   # one thread per four elements
    assert eb.echo_dropout_bwd(A, A, (1 << 40) + 1, 0.5, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_dropout_fwd(A, 8, 1.0, 1, 0, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_dropout_fwd(A, 8, -0.1, 1, 0, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_dropout_fwd(A + 4, 8, 0.5, 1, 0, A, A) == eb.ECHO_ERR_ALIGN
    assert eb.echo_dropout_bwd(A, None, 8, 0.5, A) == eb.ECHO_ERR_NULL
    assert eb.echo_dropout_bwd(A, A, 8, float("nan"), A) == eb.ECHO_ERR_SHAPE


def test_lstm_cell_rejects_bad_arguments_without_launching():
    assert eb.echo_lstm_cell_kept_bytes(128, 512, False) == 5 * 128 * 512 * 4
    assert eb.echo_lstm_cell_kept_bytes(128, 512, True) == 6 * 128 * 512 * 4
    assert eb.echo_lstm_cell_kept_bytes(0, 512, True) == 0
    assert eb.echo_lstm_cell_fwd(4, 8, A, None, A, A, A, A) == eb.ECHO_ERR_NULL
    assert eb.echo_lstm_cell_fwd(0, 8, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_lstm_cell_fwd(4, -1, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_lstm_cell_fwd(1 << 30, 1 << 30, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_lstm_cell_fwd(1 << 20, (1 << 18) + 1, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE   # B H beyond 2^38
    assert eb.echo_lstm_cell_bwd(1 << 20, (1 << 18) + 1, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_lstm_cell_fwd(4, 8, A, A, A + 4, A, A, A) == eb.ECHO_ERR_ALIGN
    assert eb.echo_lstm_cell_bwd(4, 8, None, A, A, A, A, A) == eb.ECHO_ERR_NULL
    assert eb.echo_lstm_cell_bwd(4, 8, A, A + 8, A, A, A, A) == eb.ECHO_ERR_ALIGN
    assert eb.echo_lstm_cell_fwd_stash(4, 8, A, A, A, A, A, A, None) == eb.ECHO_ERR_NULL
    assert eb.echo_lstm_cell_bwd_stash(4, 8, A, A, A, None, A, A, A) == eb.ECHO_ERR_NULL


def test_headers_are_plain_c():
    """Every public header compiles on its own as C99 (no C++ or HIP types in the boundary)."""
    import glob
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc here")
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    headers = sorted(glob.glob(os.path.join(inc, "*.h")))
    assert len(headers) >= 3
    for h in headers:
        r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", "-"],
                           input=f'#include "{h}"\n', text=True, capture_output=True)
        assert r.returncode == 0, (h, r.stderr)


def test_step_entry_points_validate():
    one = eb.make_desc(4, 1, 7, 16, 16)
    assert eb.echo_attn_step_bwd(one, A, A, A, A, A, A, A, A, A, A, None) == eb.ECHO_ERR_NULL
    assert eb.echo_attn_step_bwd(one, A, A, A, A, A, A, A, A, A, A + 4, A) == eb.ECHO_ERR_ALIGN
    assert eb.echo_attn_step_bwd(eb.make_desc(4, 2, 7, 16, 16), A, A, A, A, A, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_attn_step_bwd(eb.make_desc(4, 1, 8193, 16, 16), A, A, A, A, A, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_attn_step_fwd(one, A, A, A, A, A, A, None) == eb.ECHO_ERR_NULL
    assert eb.echo_attn_step_fwd(eb.make_desc(4, 3, 7, 16, 16), A, A, A, A, A, A, A) == eb.ECHO_ERR_SHAPE
    assert eb.echo_attn_step_finish(one, None, A) == eb.ECHO_ERR_NULL
    assert eb.echo_attn_step_finish(one, A, A + 8) == eb.ECHO_ERR_ALIGN
