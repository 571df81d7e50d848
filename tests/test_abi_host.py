"""Host-side checks that need no GPU: the library loads, exports the declared C ABI, and validates arguments."""
import ctypes
import os
import re

import pytest

from paper_2403_12422_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "jetfire.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(jf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = _declared_symbols()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTED_SYMBOLS) == names     # the binding covers the whole header, nothing more


def test_error_strings_and_workspace():
    lib = binding.load_library()
    assert lib.jf_error_string(0) == b"JF_OK"
    for code in range(1, 8):
        assert lib.jf_error_string(code).startswith(b"JF_ERR_")
    assert binding.jf_workspace_bytes(binding.JF_OP_LAYERNORM_BWD, 4096, 768, 0, 32) == 128 * 2 * 768 * 4 + 4096 * 2 * 4
    assert binding.jf_workspace_bytes(binding.JF_OP_LAYERNORM_BWD, 4096, 768, 0, 64) == 128 * 2 * 768 * 4 + 4096 * 2 * 4
    assert binding.jf_workspace_bytes(binding.JF_OP_LAYERNORM_BWD, 1 << 20, 3072, 0, 128) == 512 * 2 * 3072 * 4 + (1 << 20) * 2 * 4 * 2
    assert binding.jf_workspace_bytes(binding.JF_OP_LINEAR_FWD, 4096, 768, 3072, 32) == 0
    assert binding.jf_workspace_bytes(binding.JF_OP_LAYERNORM_BWD, 4096, 768, 0, 48) == 0


FAKE = ctypes.c_void_p(0x10000)        # aligned, never dereferenced: validation fails before any launch
ODD = ctypes.c_void_p(0x10004)


def test_argument_validation_returns_codes_without_launching():
    lib = binding.load_library()
    N, C, D = 64, 64, 64
    lin = lambda **kw: lib.jf_linear_fwd(kw.get("X", FAKE), FAKE, FAKE, FAKE, kw.get("N", N), kw.get("C", C), D,
                                         kw.get("block", 32), kw.get("Y", FAKE), kw.get("SY", FAKE), None, None, 0, None)
    assert lin(X=None) == 1                                # JF_ERR_NULL
    assert lin(Y=None) == 1
    assert lin(N=0) == 2                                   # JF_ERR_SHAPE: empty
    assert lin(N=48) == 2                                  # not a multiple of block
    assert lin(C=(1 << 24) + 32) == 2                      # above the supported maximum
    assert lin(N=1 << 24, C=1 << 24) == 2                  # more than 2^40 elements in one matrix
    assert lin(block=48) == 3                              # JF_ERR_BLOCK
    assert lin(X=ODD) == 4                                 # JF_ERR_ALIGN
    # wgrad needs at least one output, and codes/scales come together
    w = lambda dW, SdW, f: lib.jf_linear_wgrad(FAKE, FAKE, FAKE, FAKE, N, C, D, 32, dW, SdW, f, None, 0, None)
    assert w(None, None, None) == 1
    assert w(FAKE, None, None) == 1
    # quantizer
    qz = lambda **kw: lib.jf_quantize_block(kw.get("x", FAKE), kw.get("dt", 0), kw.get("rows", 64), 64, kw.get("ldx", 64),
                                            32, FAKE, 64, FAKE, kw.get("qT", None), 64, kw.get("sT", None), None)
    assert qz(x=None) == 1
    assert qz(dt=5) == 7                                   # JF_ERR_DTYPE
    assert qz(rows=33) == 2
    assert qz(ldx=32) == 2
    assert qz(qT=FAKE) == 1                                # qT without sT
    # element-wise ops and the LayerNorm-backward workspace
    assert lib.jf_gelu_q(FAKE, FAKE, 64, 65, 32, FAKE, FAKE, None) == 2
    assert lib.jf_gelu_q(FAKE, FAKE, 1 << 24, 1 << 24, 32, FAKE, FAKE, None) == 2
    assert lib.jf_gelu_q_bwd(None, FAKE, FAKE, FAKE, 64, 64, 32, FAKE, FAKE, None) == 1
    assert lib.jf_layernorm_q(FAKE, FAKE, None, FAKE, ctypes.c_float(1e-5), 64, 64, 32, FAKE, FAKE, FAKE, FAKE, None) == 1
    assert lib.jf_layernorm_q_bwd(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, 64, 32, FAKE, FAKE, FAKE, FAKE, FAKE, 16, None) == 5
    assert lib.jf_dropout_q(FAKE, FAKE, None, ctypes.c_float(0.1), 64, 64, 32, FAKE, FAKE, None) == 1
    assert lib.jf_dropout_q(FAKE, FAKE, FAKE, ctypes.c_float(1.0), 64, 64, 32, FAKE, FAKE, None) == 2
    assert lib.jf_dequantize_block(FAKE, FAKE, 64, 64, 32, FAKE, 2, 64, None) == 7
    assert lib.jf_dequantize_block(FAKE, FAKE, 64, 64, 32, FAKE, 1, 32, None) == 2
    assert lib.jf_add_q(FAKE, FAKE, None, FAKE, 64, 64, 32, FAKE, FAKE, None, None, None) == 1
    assert lib.jf_add_q(FAKE, FAKE, FAKE, FAKE, 64, 64, 32, FAKE, FAKE, FAKE, None, None) == 1      # partials come together
    assert lib.jf_add_q(FAKE, FAKE, FAKE, FAKE, 64, 80, 32, FAKE, FAKE, None, None, None) == 2
    assert lib.jf_layernorm_q_partials(FAKE, FAKE, None, FAKE, FAKE, FAKE, ctypes.c_float(1e-5), 64, 64, 32, FAKE, FAKE, FAKE,
                                       FAKE, None) == 1
    assert lib.jf_debug_linear_partials(0, FAKE, FAKE, 64, 64, 64, 32, 2, FAKE, None) == 2   # kb out of range
    assert lib.jf_debug_linear_partials(3, FAKE, FAKE, 64, 64, 64, 32, 0, FAKE, None) == 2


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(binding.JetfireError):
        binding.jf_quantize_block(torch.zeros(64, 64), 32)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU program: asking for more exits with a message before anything touches a GPU."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in (res.stderr + res.stdout)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No fallback: without the built shared object the first call raises and names the build step."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libjetfire.so"))
    with pytest.raises(binding.JetfireError, match="no CPU fallback"):
        binding.load_library()
    with pytest.raises(binding.JetfireError):
        binding.jf_workspace_bytes(binding.JF_OP_LAYERNORM_BWD, 64, 64, 0, 32)


def test_nothing_in_the_product_imports_the_oracle():
    """The oracle is test infrastructure: the package itself never imports it."""
    pkg = os.path.join(ROOT, "paper_2403_12422_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "oracle/" not in text, f


def test_oracle_shares_nothing_with_the_product():
    """The oracle neither imports the package nor includes its headers or kernels."""
    odir = os.path.join(ROOT, "oracle")
    for f in os.listdir(odir):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(odir, f)).read()
            assert "paper_2403_12422_amd" not in text and "jetfire.h" not in text and "csrc" not in text, f


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    """jf_layernorm_q_bwd_static validates like jf_layernorm_q_bwd and refuses problems whose partial rows exceed
    the static scratch, before anything is looked up or launched."""
    lib = binding.load_library()
    call = lambda N, C, block=32, dY=FAKE: lib.jf_layernorm_q_bwd_static(dY, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, N, C, block,
                                                                       FAKE, FAKE, FAKE, FAKE, None)
    assert call(64, 64, dY=None) == 1                      # JF_ERR_NULL
    assert call(48, 64) == 2                               # JF_ERR_SHAPE
    assert call(64, 64, block=48) == 3                     # JF_ERR_BLOCK
    assert call(64, 64, dY=ODD) == 4                       # JF_ERR_ALIGN
    scratch = 8 << 20
    assert binding.jf_workspace_bytes(binding.JF_OP_LAYERNORM_BWD, 16384, 4096, 0, 64) > scratch       # 512 partial rows of 32 KiB
    assert call(16384, 4096, block=64) == 5                # JF_ERR_WORKSPACE
    assert binding.jf_workspace_bytes(binding.JF_OP_LAYERNORM_BWD, 1 << 20, 768, 0, 32) > scratch      # 8 bytes per row
    assert call(1 << 20, 768) == 5


def test_linear_bwd_validates_like_dgrad_and_wgrad():
    lib = binding.load_library()
    N, C, D = 64, 64, 64

    def call(dY=FAKE, X=FAKE, dX=FAKE, SdX=FAKE, dW=FAKE, SdW=FAKE, dWf=None, N=N, block=32):
        return lib.jf_linear_bwd(dY, FAKE, FAKE, FAKE, X, FAKE, N, C, D, block, dX, SdX, None, dW, SdW, dWf, None, 0, None)
    assert call(dY=None) == 1                              # JF_ERR_NULL
    assert call(X=None) == 1
    assert call(dX=None) == 1                              # the input gradient's INT8 output is required ...
    assert call(dW=None, SdW=None) == 1                    # ... and the weight gradient needs at least one output
    assert call(dW=FAKE, SdW=None) == 1                    # codes and scales come together
    assert call(N=48) == 2                                 # JF_ERR_SHAPE
    assert call(block=48) == 3                             # JF_ERR_BLOCK
    assert call(X=ODD) == 4                                # JF_ERR_ALIGN
