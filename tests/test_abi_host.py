"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, the host-only slice strategy equals the oracle, and argument validation
returns error codes before any device work."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2408_11500_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2408_11500_amd import build
        build.build(verbose=False)
    return binding.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "slicegcn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slicegcn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert len(names) == 24 and set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_slice_strategy_matches_oracle(L):
    for d in range(1, 80):
        for p in range(1, d + 1):
            assert binding.slicegcn_slice_strategy(d, p) == oracle.slice_strategy(d, p)
    for d, p, s in [(100, 4, 0.5), (100, 4, 1.5), (301, 3, 1.0), (602, 2, 1.0), (7, 2, 1.7)]:
        assert binding.slicegcn_slice_strategy(d, p, s) == oracle.slice_strategy(d, p, s)


@pytest.mark.parametrize("args", [(0, 1, 1.0), (4, 0, 1.0), (4, 5, 1.0), (4, 2, 0.0), (4, 2, -1.0), (4, 2, 0.1), (4, 2, 3.0)])
def test_slice_strategy_rejects(L, args):
    with pytest.raises(binding.SliceGCNError) as e:
        binding.slicegcn_slice_strategy(*args)
    assert e.value.status == binding.EINVAL
    with pytest.raises(ValueError):
        oracle.slice_strategy(*args)


def test_cosine_lr_matches_oracle(L):
    for t in range(0, 51, 5):
        assert abs(binding.slicegcn_cosine_lr(0.01, 1e-4, t, 50) - oracle.cosine_lr(0.01, 1e-4, t, 50)) < 1e-15
    assert binding.slicegcn_cosine_lr(0.01, 0.0, 3, 0) == 0.01


def test_null_and_size_errors_return_codes(L):
    h = ctypes.c_void_p(0)
    assert L.slicegcn_build_norm_csr(None, None, 0, 0, 3, None, ctypes.byref(h)) == binding.EINVAL      # n_nodes < 1
    assert L.slicegcn_build_norm_csr(None, None, 5, 10, 3, None, ctypes.byref(h)) == binding.EINVAL     # NULL edges
    assert L.slicegcn_build_norm_csr(None, None, 0, 10, 8, None, ctypes.byref(h)) == binding.EINVAL     # unknown flag
    assert L.slicegcn_build_norm_csr(None, None, 0, 1 << 31, 3, None, ctypes.byref(h)) == binding.ERANGE
    assert L.slicegcn_build_norm_csr(None, None, 0, 10, 3, None, None) == binding.EINVAL
    assert L.slicegcn_spmm_slice(None, 0, None, 4, 4, None, 4, None) == binding.EINVAL
    assert L.slicegcn_slice_feature(None, 4, 4, 0, 2, None, 2, None) == binding.EINVAL
    assert L.slicegcn_graph_destroy(None) == binding.OK
    assert L.slicegcn_layer_bwd_workspace_bytes(0, None, 1) == 0
    assert b"NULL" in L.slicegcn_last_error()
    assert L.slicegcn_strerror(binding.EWORKSPACE) == b"workspace missing or too small"
    assert L.slicegcn_strerror(-99) == b"unknown status"


def test_workspace_formula(L):
    # partial sums: ceil(n / 1024) row blocks x (2*w_in*w_out + 2*w_out) floats, 256-byte rounded,
    # plus an n x roundup4(w_in) fp32 staging matrix when the input gradient is wanted
    n, w_in, w_out = 5000, 25, 64
    part = -(-(5 * (2 * w_in * w_out + 2 * w_out) * 4) // 256) * 256
    assert binding.slicegcn_layer_bwd_workspace_bytes(n, w_in, w_out, False) == part
    assert binding.slicegcn_layer_bwd_workspace_bytes(n, w_in, w_out, True) == part + -(-(n * 28 * 4) // 256) * 256
