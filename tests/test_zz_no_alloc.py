"""The entry point that allocates nothing (ziplm_module_error_static) against the entry point it is a variant of
(ziplm_module_error), through the C ABI: same kernels, so the whole-module error tr(W (H + lambda I) W^T) must come out
bit for bit, on two calls in a row that share the library's built-in scratch array, the second on a smaller layer.
Also against the oracle at the bar of the regular test, and the size limit."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2302_04089_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def z():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2302_04089_amd import ziplm
    ziplm.lib()
    return ziplm


def _layer(oracle, m, d, n, seed):
    spec = workloads.small(m, d, 1, n, x_kind="gelu", seed=seed)
    X = workloads.make_X(spec)
    W32 = workloads.make_W(spec)
    H32 = oracle.hessian(X, 2.0).astype(np.float32)
    return W32, H32


def test_static_scratch_entry_point_equals_the_workspace_one(z, oracle):
    L = z.lib()
    lam = 3.5
    outs = []
    for m, d, n, seed in ((300, 520, 1500, 91), (40, 130, 400, 92)):       # the second call is the smaller one
        W32, H32 = _layer(oracle, m, d, n, seed)
        W = torch.from_numpy(W32).cuda()
        H = torch.from_numpy(H32).cuda()
        want = torch.zeros(1, dtype=torch.float64, device="cuda")
        got = torch.zeros(1, dtype=torch.float64, device="cuda")
        ws = torch.empty(max(z.ziplm_module_error_workspace_bytes(m, d), 256), dtype=torch.uint8, device="cuda")
        rc = L.ziplm_module_error(W.data_ptr(), H.data_ptr(), m, d, lam, want.data_ptr(), ws.data_ptr(), ws.numel(), None)
        assert rc == 0
        rc = L.ziplm_module_error_static(W.data_ptr(), H.data_ptr(), m, d, lam, got.data_ptr(), None)
        assert rc == 0
        torch.cuda.synchronize()
        assert got.item() == want.item(), "static %r vs workspace %r" % (got.item(), want.item())
        ref = oracle.module_error(W32, H32, lam)
        assert abs(got.item() - ref) <= 1e-5 * abs(ref)
        outs.append(got.item())
    assert outs[0] != outs[1]


def test_static_scratch_entry_point_limits_and_arguments(z):
    L = z.lib()
    one = ctypes.c_void_p(256)      # never dereferenced: validation fails first
    assert L.ziplm_module_error_static_max_tiles() == 4096
    assert L.ziplm_module_error_static(None, one, 2, 8, 0.0, one, None) == z.ERR_INVALID_ARG
    assert L.ziplm_module_error_static(one, one, 2, 8, -1.0, one, None) == z.ERR_INVALID_ARG
    assert L.ziplm_module_error_static(one, one, 128 * 65, 128 * 64, 0.0, one, None) == z.ERR_UNSUPPORTED    # 4160 tiles
    # exactly at the limit the request is accepted by the size check (64 x 64 tiles); not run here: 67 million weights
    assert z.ziplm_module_error_workspace_bytes(128 * 64, 128 * 64) == 4096 * 8
