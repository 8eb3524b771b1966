"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/bb.h declares, and rejects bad arguments before touching
the device."""
import ctypes
import os
import re

import pytest

import paper_2505_07829_amd as bb
from paper_2505_07829_amd import build as bb_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    bb_build.build(force=False)
    return bb.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "bb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bb_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert "bb_rmsnorm_swiglu_ffn" in names and "bb_layernorm_matmul" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(bb.binding.EXPORTS) == names


def test_version_and_strings(lib):
    assert bb.bb_version() == 100
    assert bb.status_string(0) == "ok"
    for s in range(-9, 0):
        assert bb.status_string(s) not in ("ok", "unknown status")
    assert bb.status_string(-99) == "unknown status"


A = 0x10000   # fake, aligned, non-overlapping "device addresses": never dereferenced


def ffn(lib, X=A, g=2 * A, W1=3 * A, W3=4 * A, W2=5 * A, Y=6 * A, M=4, D=64, F=128, eps=1e-6, fn=None):
    fn = fn or lib.bb_rmsnorm_swiglu_ffn
    return fn(X, g, W1, W3, W2, Y, M, D, F, eps, None)


def ln(lib, X=A, ga=2 * A, be=3 * A, W=4 * A, Y=6 * A, M=4, D=64, N=128, eps=1e-6, fn=None):
    fn = fn or lib.bb_layernorm_matmul
    return fn(X, ga, be, W, Y, M, D, N, eps, None)


@pytest.mark.parametrize("unfused", ["", "_unfused", "_t"])
def test_ffn_argument_errors(lib, unfused):
    fn = getattr(lib, "bb_rmsnorm_swiglu_ffn" + unfused)
    assert ffn(lib, fn=fn, M=0) == 0                       # empty input: nothing to do
    assert ffn(lib, fn=fn, M=0, X=None, Y=None) == 0
    assert ffn(lib, fn=fn, M=-1) == -2
    assert ffn(lib, fn=fn, D=0) == -2
    assert ffn(lib, fn=fn, D=60) == -2                     # not a multiple of 8
    assert ffn(lib, fn=fn, F=130) == -2
    assert ffn(lib, fn=fn, D=(1 << 24) + 8) == -2
    for k in ("X", "g", "W1", "W3", "W2", "Y"):
        assert ffn(lib, fn=fn, **{k: None}) == -1
        assert ffn(lib, fn=fn, **{k: A * 7 + 2}) == -3     # misaligned
    assert ffn(lib, fn=fn, eps=-1.0) == -4
    assert ffn(lib, fn=fn, eps=float("nan")) == -4
    assert ffn(lib, fn=fn, eps=float("inf")) == -4
    assert ffn(lib, fn=fn, Y=A) == -5                      # in place
    assert ffn(lib, fn=fn, Y=A + 16) == -5                 # partial overlap with X
    assert ffn(lib, fn=fn, Y=5 * A + 64) == -5             # overlap with W2


@pytest.mark.parametrize("unfused", ["", "_unfused", "_t"])
def test_ln_argument_errors(lib, unfused):
    fn = getattr(lib, "bb_layernorm_matmul" + unfused)
    assert ln(lib, fn=fn, M=0) == 0
    assert ln(lib, fn=fn, M=-3) == -2
    assert ln(lib, fn=fn, N=12) == -2
    for k in ("X", "ga", "be", "W", "Y"):
        assert ln(lib, fn=fn, **{k: None}) == -1
        assert ln(lib, fn=fn, **{k: A * 9 + 4}) == -3
    assert ln(lib, fn=fn, eps=-1e-9) == -4
    assert ln(lib, fn=fn, Y=4 * A) == -5


def attn(lib, Q=A, K=2 * A, V=3 * A, O=6 * A, B=2, M=16, N=16, d=64, dv=64):
    return lib.bb_attention(Q, K, V, O, B, M, N, d, dv, None)


def test_attention_argument_errors(lib):
    assert attn(lib, B=0) == 0 and attn(lib, M=0) == 0      # nothing to do
    assert attn(lib, B=0, Q=None, O=None) == 0
    assert attn(lib, B=-1) == -2 and attn(lib, M=-1) == -2
    assert attn(lib, N=0) == -2                             # softmax over no keys
    for bad in (0, 32, 96, 72, 256):
        assert attn(lib, d=bad) == -2
        assert attn(lib, dv=bad) == -2
    assert attn(lib, M=(1 << 24) + 1) == -2
    assert attn(lib, N=1 << 24) == -2
    assert attn(lib, B=1 << 30, M=1024) == -2               # more workgroups than a launch takes
    for k in ("Q", "K", "V", "O"):
        assert attn(lib, **{k: None}) == -1
        assert attn(lib, **{k: A * 7 + 2}) == -3
    assert attn(lib, O=A) == -5
    assert attn(lib, O=2 * A + 32) == -5
    assert attn(lib, O=3 * A - 64) == -5                    # tail of O runs into V


@pytest.mark.parametrize("suffix", ["", "_t"])
def test_residual_argument_errors_and_aliasing(lib, suffix):
    fn = getattr(lib, "bb_rmsnorm_swiglu_ffn_residual" + suffix)

    def call(X=A, g=2 * A, W1=3 * A, W3=4 * A, W2=5 * A, R=7 * A, Y=6 * A, M=4, D=64, F=128, eps=1e-6):
        return fn(X, g, W1, W3, W2, R, Y, M, D, F, eps, None)
    assert call(M=0) == 0 and call(M=0, R=None) == 0
    assert call(M=-1) == -2 and call(D=60) == -2 and call(eps=-1.0) == -4
    for k in ("X", "g", "W1", "W3", "W2", "R", "Y"):
        assert call(**{k: None}) == -1
        assert call(**{k: A * 9 + 2}) == -3
    assert call(Y=A) == -5                          # over X, not in place with R
    assert call(Y=7 * A + 16) == -5                 # partial overlap with R
    assert call(Y=5 * A) == -5                      # over a weight
    assert call(R=A, Y=A + 16) == -5                # R is X, Y overlaps both partially


def test_tune_argument_errors(lib):
    import ctypes as C
    f = lib.bb_rmsnorm_swiglu_ffn_tune
    args = [A, 2 * A, 3 * A, 4 * A, 5 * A, 6 * A, 4, 64, 128, 1e-6, None]
    assert f(*args, 0, None, None) == -2                    # reps out of range
    assert f(*args, 1001, None, None) == -2
    bad = list(args); bad[6] = 0
    assert f(*bad, 3, None, None) == -2                     # nothing to measure on an empty input
    bad = list(args); bad[0] = None
    assert f(*bad, 3, None, None) == -1
    bad = list(args); bad[5] = A
    assert f(*bad, 3, None, None) == -5
    h = lib.bb_layernorm_matmul_tune
    largs = [A, 2 * A, 3 * A, 4 * A, 6 * A, 4, 64, 128, 1e-6, None]
    assert h(*largs, 0, None, None) == -2
    bad = list(largs); bad[7] = 12
    assert h(*bad, 3, None, None) == -2
    assert lib.bb_tuned_variant(0, 4, 64, 128) == 0         # nothing recorded
    assert lib.bb_tune_clear() == 0


def test_variant_and_workspace_queries(lib):
    assert bb.bb_get_variant() in (0, 1, 2)
    old = bb.bb_get_variant()
    with pytest.raises(bb.BBError):
        bb.bb_set_variant(6)
    bb.bb_set_variant(bb.VARIANT_NEST)
    assert bb.bb_get_variant() == bb.VARIANT_NEST
    bb.bb_set_variant(bb.VARIANT_UNFUSED)
    assert bb.bb_get_variant() == bb.VARIANT_UNFUSED
    bb.bb_set_variant(bb.VARIANT_PRESCALE)
    assert bb.bb_get_variant() == bb.VARIANT_PRESCALE
    bb.bb_set_variant(bb.VARIANT_SNAPSHOT1)
    assert bb.bb_get_variant() == bb.VARIANT_SNAPSHOT1
    bb.bb_set_variant(old)
    # hidden (M*F bf16) must fit; invalid sizes give 0
    assert bb.bb_workspace_bytes(bb.OP_FFN, 2048, 4096, 11008) >= 2048 * 11008 * 2
    assert bb.bb_workspace_bytes(bb.OP_FFN, 16, 4096, 11008) >= 16 * 4096 * 4 + 2 * 2 * 16 * 11008 * 4
    assert bb.bb_workspace_bytes(bb.OP_LN, 8192, 4096, 16384) >= 2 * 16384 * 4
    assert bb.bb_workspace_bytes(bb.OP_FFN_UNFUSED, 64, 256, 704) >= 64 * 256 * 2 + 3 * 64 * 704 * 2
    assert bb.bb_workspace_bytes(bb.OP_FFN, 4, 7, 8) == 0
    assert bb.bb_workspace_bytes(99, 4, 8, 8) == 0
    assert lib.bb_set_workspace(ctypes.c_void_p(A + 8), 1024) == -7     # misaligned
    assert lib.bb_set_workspace(None, 1024) == -7
    assert lib.bb_set_workspace(None, 0) == 0


def test_calibration_argument_errors(lib):
    assert lib.bb_calib_copy(None, A, 1024, None) == -1
    assert lib.bb_calib_copy(A, 2 * A, 1000, None) == -3
    assert lib.bb_calib_copy(A, A + 512, 1024, None) == -5
    assert lib.bb_calib_read(A, 1024, None, None) == -1
    assert lib.bb_calib_mfma(0, 10, A, None) == -2
    assert lib.bb_calib_mfma_data(None, 4, 10, A, None) == -1
    assert lib.bb_calib_mfma_data(A + 8, 4, 10, A, None) == -3
    assert lib.bb_calib_mfma_data(A, 4, 0, A, None) == -2
