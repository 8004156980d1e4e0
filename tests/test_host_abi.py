"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and rejects bad arguments
before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2409_15373_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2409_15373_amd import build
        build.build()
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "jfa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(jfa_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2409_15373_amd import binding
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_workspace_depend_on_B_only(lib):
    from paper_2409_15373_amd import binding
    assert binding.jfa_version() >= 100
    a = binding.jfa_workspace_bytes(512, 4096, 8, 128)
    assert a == binding.jfa_workspace_bytes(512, 1 << 20, 1, 32, backward=True)     # no max_len / H / D term
    assert a <= 64 * 4 + 2 * (2 * 512 + 1) * 4 + 1024
    assert binding.jfa_workspace_bytes(0, 10, 1, 32) == 0


@pytest.mark.parametrize("fn", ["jfa_forward", "jfa_forward_f32", "jfa_forward_causal", "jfa_forward_causal_f32"])
def test_forward_argument_errors(lib, fn):
    from paper_2409_15373_amd import binding
    f = getattr(lib, fn)
    assert f(None, None, None, None, -1, 8, 1, 32, None, None, None) == binding.JFA_ERR_INVALID_ARG
    assert "negative" in binding.jfa_last_error()
    assert f(None, None, None, None, 1, -8, 1, 32, None, None, None) == binding.JFA_ERR_INVALID_ARG
    assert f(None, None, None, None, 1, 8, 0, 32, None, None, None) == binding.JFA_ERR_INVALID_ARG
    assert f(None, None, None, None, 1, 8, 1, 48, None, None, None) == binding.JFA_ERR_UNSUPPORTED
    assert "D = 48" in binding.jfa_last_error()
    assert f(None, None, None, None, 1, 8, 1, 64, None, None, None) == binding.JFA_ERR_INVALID_ARG
    assert "null" in binding.jfa_last_error()
    assert f(16, 16, 16, 16, 1, 8, 1, 64, 16, 8, None) == binding.JFA_ERR_INVALID_ARG      # lse misaligned
    assert "aligned" in binding.jfa_last_error()
    assert f(None, None, None, None, 0, 8, 1, 64, None, None, None) == binding.JFA_OK        # B == 0: nothing to do


@pytest.mark.parametrize("fn", ["jfa_backward", "jfa_backward_f32", "jfa_backward_causal", "jfa_backward_causal_f32"])
def test_backward_argument_errors(lib, fn):
    from paper_2409_15373_amd import binding
    f = getattr(lib, fn)
    n = [None] * 7
    assert f(*n, -1, 8, 1, 32, None, None, None, None, None) == binding.JFA_ERR_INVALID_ARG
    assert f(*n, 1, 8, 1, 96, None, None, None, None, None) == binding.JFA_ERR_UNSUPPORTED
    assert f(*n, 1, 8, 1, 128, None, None, None, None, None) == binding.JFA_ERR_INVALID_ARG
    assert f(*n, 0, 8, 1, 128, None, None, None, None, None) == binding.JFA_OK


def test_schedule_and_check_argument_errors(lib):
    from paper_2409_15373_amd import binding
    assert lib.jfa_build_schedule(None, 4, 128, None, None, None) == binding.JFA_ERR_INVALID_ARG
    assert lib.jfa_build_schedule(16, 4, 100, 16, 16, None) == binding.JFA_ERR_INVALID_ARG
    assert "multiple of 32" in binding.jfa_last_error()
    assert lib.jfa_check_offsets(16, 4, 10, None, None) == binding.JFA_ERR_INVALID_ARG


def test_unfused_conversion_and_feature_operator_argument_errors(lib):
    from paper_2409_15373_amd import binding
    OK, BAD, UNS = binding.JFA_OK, binding.JFA_ERR_INVALID_ARG, binding.JFA_ERR_UNSUPPORTED
    assert lib.jfa_square_offsets(None, 4, None, None) == BAD
    assert lib.jfa_square_offsets(None, -1, None, None) == BAD
    assert lib.jfa_unfused_scores(None, None, None, None, 1, 8, 1, 48, None, None) == UNS
    assert lib.jfa_unfused_scores(None, None, None, None, 1, 8, 1, 64, None, None) == BAD
    assert lib.jfa_unfused_scores(None, None, None, None, 0, 8, 1, 64, None, None) == OK
    assert lib.jfa_unfused_softmax(None, None, 1, 8, 0, None, None) == BAD                  # H = 0
    assert lib.jfa_unfused_apply(None, None, None, None, -2, 8, 1, 64, None, None) == BAD
    assert lib.jfa_unfused_product(None, None, None, None, 1, 8, 1, 64, 1.0, None, None) == BAD
    assert lib.jfa_unfused_product(None, None, None, None, 1, 8, 1, 50, 1.0, None, None) == UNS
    assert lib.jfa_unfused_softmax_backward(None, None, None, 1, 8, 2, 1.0, None, None) == BAD
    assert lib.jfa_unfused_softmax_backward(None, None, None, 0, 8, 2, 1.0, None, None) == OK
    assert lib.jfa_unfused_apply_transposed(16, 16, 16, 16, 1, 8, 1, 64, 8, None) == BAD     # out misaligned
    # conversions: row_bytes must be a positive multiple of 16; null and misaligned tensors are refused
    assert lib.jfa_jagged_to_dense(16, 16, 2, 8, 24, 0, 16, None) == UNS
    assert "multiple of 16" in binding.jfa_last_error()
    assert lib.jfa_jagged_to_dense(None, 16, 2, 8, 32, 0, 16, None) == BAD
    assert lib.jfa_jagged_to_dense(8, 16, 2, 8, 32, 0, 16, None) == BAD
    assert "aligned" in binding.jfa_last_error()
    assert lib.jfa_dense_to_jagged(16, 16, 2, -1, 32, 16, None) == BAD
    assert lib.jfa_dense_to_jagged(None, None, 0, 8, 32, None, None) == OK                  # B == 0: nothing to do
    assert lib.jfa_jagged_to_dense(None, None, 3, 0, 32, 0, None, None) == OK               # max_len == 0: an empty dense tensor
    # feature operators: D and T each one of 32, 64, 128
    assert lib.jfa_jagged_dense_bmm(None, None, None, 1, 8, 64, 48, None, None) == UNS
    assert "T = 48" in binding.jfa_last_error()
    assert lib.jfa_jagged_dense_bmm(None, None, None, 1, 8, 16, 64, None, None) == UNS
    assert lib.jfa_jagged_jagged_bmm(None, None, None, 1, 8, 64, 64, None, None) == BAD
    assert "null" in binding.jfa_last_error()
    assert lib.jfa_jagged_jagged_bmm(None, None, None, 0, 8, 64, 64, None, None) == OK
    assert lib.jfa_jagged_softmax(None, None, 1, 8, 96, None, None) == UNS
    assert lib.jfa_jagged_softmax_backward(16, 16, 16, 1, 8, 64, 8, None) == BAD            # dx misaligned


@pytest.mark.parametrize("suffix", ["", "_f32"])
def test_cross_attention_argument_errors(lib, suffix):
    from paper_2409_15373_amd import binding
    OK, BAD, UNS = binding.JFA_OK, binding.JFA_ERR_INVALID_ARG, binding.JFA_ERR_UNSUPPORTED
    fwd, bwd = getattr(lib, "jfa_forward_cross" + suffix), getattr(lib, "jfa_backward_cross" + suffix)
    assert fwd(16, 16, 16, 16, None, 1, 8, 8, 1, 64, 16, 16, None) == BAD                    # offsets_kv is null
    assert "offsets_kv" in binding.jfa_last_error()
    assert fwd(16, 16, 16, 16, 8, 1, 8, 8, 1, 64, 16, 16, None) == BAD                       # offsets_kv misaligned
    assert fwd(16, 16, 16, 16, 16, 1, 8, -8, 1, 64, 16, 16, None) == BAD
    assert "max_len_kv" in binding.jfa_last_error()
    assert fwd(16, 16, 16, 16, 16, 1, 8, 8, 1, 80, 16, 16, None) == UNS
    assert fwd(None, None, None, None, None, 0, 8, 8, 1, 64, None, None, None) == OK         # B == 0: nothing to do
    n = [16] * 6
    assert bwd(*n, 16, None, 1, 8, 8, 1, 64, 16, 16, 16, 16, None) == BAD
    assert bwd(*n, 16, 16, -1, 8, 8, 1, 64, 16, 16, 16, 16, None) == BAD
    assert bwd(*n, 16, 16, 1, 8, 8, 0, 64, 16, 16, 16, 16, None) == BAD                      # H = 0
    assert bwd(*([None] * 8), 0, 8, 8, 1, 64, None, None, None, None, None) == OK


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2409_15373_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.load()
