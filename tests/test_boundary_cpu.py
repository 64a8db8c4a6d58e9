"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments
before touching the GPU.  No compute calls: runs without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2503_16672_amd", "libffn24.so")
HEADER = os.path.join(ROOT, "include", "ffn24.h")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libffn24.so not built (python -m paper_2503_16672_amd.build)")


def _declared():
    src = open(HEADER).read()
    return re.findall(r"FFN24_API\s+(?:const\s+)?\w+\*?\s+(\w+)\s*\(", src)


def test_header_symbols_are_exported():
    names = _declared()
    assert len(names) == 32 and "ffn24_fwd" in names and "sparsify24" in names
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_names():
    from paper_2503_16672_amd import ffn24
    assert sorted(ffn24.EXPORTS) == sorted(_declared())
    ffn24.lib()


def test_strerror():
    from paper_2503_16672_amd import ffn24
    assert ffn24.strerror(0) == "ok"
    assert "NULL" in ffn24.strerror(-1)
    assert "unknown" in ffn24.strerror(-99)


def test_argument_validation_without_gpu():
    from paper_2503_16672_amd import ffn24
    L = ffn24.lib()
    a16 = 0x1000
    # sparsify24: cols not a multiple of 8, negative rows, NULL, misaligned, unsupported dtype; rows == 0 is a no-op
    assert L.sparsify24(a16, 4, 12, 0, a16, a16, None) == -2
    assert L.sparsify24(a16, -1, 16, 0, a16, a16, None) == -2
    assert L.sparsify24(None, 4, 16, 0, a16, a16, None) == -1
    assert L.sparsify24(a16 + 2, 4, 16, 0, a16, a16, None) == -3
    assert L.sparsify24(a16, 4, 16, 2, a16, a16, None) == -4
    assert L.sparsify24(a16, 4, 24, 1, a16, a16, None) == -2          # e4m3 input: cols a multiple of 16
    assert L.sparsify24_quantise(a16, 4, 16, ctypes.c_float(0.0), a16, a16, None) == -2
    assert L.sparsify24_quantise(a16, 4, 12, ctypes.c_float(1.0), a16, a16, None) == -2
    assert L.sparsify24_quantise(None, 4, 16, ctypes.c_float(1.0), a16, a16, None) == -1
    assert L.sparsify24(None, 0, 16, 0, None, None, None) == 0
    # spmm24 shape rules
    assert L.spmm24(a16, a16, a16, 256, 256, 32, a16, None) == -2
    assert L.spmm24(a16, a16, a16, 100, 256, 64, a16, None) == -2
    assert L.spmm24(a16, a16, a16 + 8, 256, 256, 64, a16, None) == -3
    assert L.spmm24(None, a16, a16, 256, 256, 64, a16, None) == -1
    # row-wise / column-wise quantisation
    assert L.quantise_e4m3(a16, 4, 16, 2, a16, a16, None) == -2 and L.quantise_e4m3(a16, 4, 12, 1, a16, a16, None) == -2
    assert L.quantise_e4m3(None, 4, 16, 1, a16, a16, None) == -1 and L.quantise_e4m3(a16 + 2, 4, 16, 1, a16, a16, None) == -3
    assert L.quantise_e4m3(None, 0, 16, 0, None, None, None) == 0
    # feature-wise
    assert L.sparsify24_featurewise(a16, a16, None, 100, 64, a16, a16, None, None) == -2
    assert L.sparsify24_featurewise(a16, a16, a16, 128, 64, a16, a16, None, None) == -1
    # context: shape and dtype rules are checked before any allocation
    h = ctypes.c_void_p()
    assert L.ffn24_ctx_create(ctypes.byref(h), 100, 512, 2048, 0, 0) == -2
    assert L.ffn24_ctx_create(ctypes.byref(h), 256, 512, 2048, 1, 1 | 8) == -4   # fp8: the split needs the row-wise recipe
    assert L.ffn24_ctx_create(ctypes.byref(h), 256, 512, 2048, 1, 1 | 32) == -4  # fp8: the token permutation too
    assert L.ffn24_bwd_rowwise(None, None, a16, a16, a16, None) == -1 and L.ffn_bwd_rowwise(None, None, a16, a16, a16, None) == -1
    assert L.ffn24_ctx_create(ctypes.byref(h), 256, 512, 2048, 2, 0) == -4
    assert L.ffn24_set_scales(None, 1.0, 1.0, 1.0, 1.0) == -1
    assert L.ffn24_ctx_create(None, 256, 512, 2048, 0, 0) == -1
    assert h.value is None
    assert L.ffn24_fwd(None, a16, a16, None, a16, a16, None) == -1
    assert L.ffn24_ctx_destroy(None) == 0
    assert L.ffn24_ctx_create(ctypes.byref(h), 256, 512, 2048, 1, 64) == -4  # telemetry is a bf16 feature
    assert L.ffn24_prepare_weights(None, a16, a16, None) == -1
    n5 = (ctypes.c_int64 * 5)()
    assert L.ffn24_get_telemetry(None, n5, 0) == -1
    use = ctypes.c_int()
    assert L.ffn24_policy_use_sparse(None, 0.9, ctypes.byref(use)) == -1


def test_binding_checks_shapes_and_dtypes_before_the_call():
    """The binding rejects tensors whose shape or element type does not match the call (the C ABI sees only pointers)."""
    import torch
    from paper_2503_16672_amd import ffn24
    ok = torch.zeros((4, 16), dtype=torch.bfloat16)
    ffn24._expect(ok, (4, 16), ffn24._BF16, "H")
    ffn24._expect(None, (4, 16), ffn24._BF16, "optional")
    with pytest.raises(ValueError, match="shape"):
        ffn24._expect(ok, (4, 8), ffn24._BF16, "H")
    with pytest.raises(ValueError, match="dtype"):
        ffn24._expect(ok.float(), (4, 16), ffn24._BF16, "H")
    with pytest.raises(ValueError, match="CUDA"):
        ffn24.sparsify24(ok)                       # right shape and type, but host memory


def test_bench_refuses_more_than_one_gpu():
    """This build is single-GPU: bench.py --gpus N with N > 1 exits with a message instead of launching anything."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_static_forward_argument_validation_without_gpu():
    """ffn24_fwd_static checks sizes against the static scratch buffer, and pointers, before it touches the GPU."""
    from paper_2503_16672_amd import ffn24
    L = ffn24.lib()
    a16 = 0x1000
    assert ffn24.static_scratch_needed(256, 256, 256) == 256 * 256 + 256 * 256 // 8 + 4 * 256 * 256
    assert ffn24.static_scratch_needed(1024, 1024, 4096) == 1024 * 4096 * 9 // 8 + 4 * 1024 * 4096
    assert ffn24.static_scratch_needed(0, 256, 256) == -1
    assert L.ffn24_fwd_static(a16, a16, None, a16, a16, 300, 256, 256, None) == -2
    assert L.ffn24_fwd_static(a16, a16, None, a16, a16, 16384, 4096, 16384, None) == -8
    assert L.ffn24_fwd_static(a16, None, None, a16, a16, 256, 256, 256, None) == -1
    assert L.ffn24_fwd_static(a16, a16, 0x1004, a16, a16, 256, 256, 256, None) == -3

