"""The C-ABI library loads and exports every symbol the header declares; the host-only
size queries behave.  No GPU needed (no kernel is launched)."""
import ctypes
import os
import re

import pytest

from paper_2602_04163_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_04163_amd import build
        build.build(verbose=False)
    return binding.load()


def _declared():
    text = open(os.path.join(ROOT, "include", "bpdq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bpdq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert sorted(names) == sorted(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_no_torch_types_in_the_abi():
    text = open(os.path.join(ROOT, "include", "bpdq.h")).read()
    assert "torch" not in text and "at::" not in text
    assert 'extern "C"' in text


def test_size_queries(lib):
    assert lib.bpdq_version() >= 100
    p = binding.make_params(2, 128, 128, 5)
    need = binding.bpdq_quantize_workspace_bytes(3584, 3584, p)
    assert need >= 3584 * 3584 * 4
    bad = binding.make_params(5, 128, 128, 5)
    assert binding.bpdq_quantize_workspace_bytes(3584, 3584, bad) == 0
    bad = binding.make_params(2, 48, 128, 5)
    assert binding.bpdq_quantize_workspace_bytes(3584, 3584, bad) == 0
    bad = binding.make_params(2, 128, 128, 5, grid=7)
    assert binding.bpdq_quantize_workspace_bytes(3584, 3584, bad) == 0
    bad = binding.make_params(2, 128, 128, 5)
    bad.coef_fp16 = 2
    assert binding.bpdq_quantize_workspace_bytes(3584, 3584, bad) == 0
    assert binding.bpdq_quantize_workspace_bytes(3584, 3584, binding.make_params(2, 128, 128, 5, coef_fp16=True)) == need
    assert binding.bpdq_quantize_workspace_bytes(8192, 8192, binding.make_params(2, 256, 128, 10)) > 0
    # four planes at group size 256 are not built
    assert binding.bpdq_quantize_workspace_bytes(8192, 8192, binding.make_params(4, 256, 256, 5)) == 0
    assert binding.bpdq_quantize_workspace_bytes(8192, 8192, binding.make_params(4, 128, 128, 5)) > 0
    assert binding.bpdq_prepare_workspace_bytes(3584) >= 3584 * 3584 * 8
    assert binding.bpdq_hessian_workspace_bytes(0, 3584) == 0
    # a full 262144-token call on a 3584-wide layer is split over the token axis (partial tiles)
    # and its activations are kept as two fp16 halves per value (as many bytes as X)
    assert binding.bpdq_hessian_workspace_bytes(262144, 3584) >= 262144 * 3584 * 4 + 105 * 256 * 256 * 4
    assert binding.bpdq_hessian_workspace_bytes(262144, 3584) % 256 == 0


def test_argument_errors_are_reported_without_a_gpu(lib):
    # invalid arguments are rejected on the host before any HIP call
    assert lib.bpdq_hessian_accumulate_f32(None, -1, 64, 64, 2.0, None, 0, None, 0, None) == -2
    assert lib.bpdq_hessian_accumulate_f32(None, 0, 6, 64, 2.0, None, 0, None, 0, None) == -3
    assert lib.bpdq_hessian_accumulate(None, -1, 64, 64, 2.0, None, 0, None, 0, None) == -2
    assert lib.bpdq_hessian_accumulate(None, 0, 6, 64, 2.0, None, 0, None, 0, None) == -3
    assert lib.bpdq_prepare(None, 64, 0.01, None, None, None, None, 0, None) == -1
    assert lib.bpdq_pack_planes(None, 4, 64, 2, None, None) == -1
    assert lib.bpdq_dequant(None, None, 4, 64, 2, 32, None, None) == -1
    assert lib.bpdq_dequant_fp16(None, None, 4, 64, 2, 32, None, None) == -1
    assert lib.bpdq_quantize_layers(None, 4, 64, None, None, None, 1, None, None, None, None, None,
                                    None, None, 0, None) == -1
    assert lib.bpdq_channel_order(None, 64, 1, None, None, 0, None) == -1
    assert lib.bpdq_gather_symmetric(None, 64, None, None, None) == -1
    assert lib.bpdq_gemv(None, None, 4, 64, 2, 32, None, None, None) == -1
    assert binding.load().bpdq_channel_order_workspace_bytes(3584) >= 3584 * 8
    assert lib.bpdq_coefs_to_fp16(None, 4, None, None) == -1
    assert lib.bpdq_coefs_to_fp16(None, 0, None, None) == 0       # nothing to convert
