"""The sublayer tail that allocates nothing (lsq_k_gemm_add_layernorm_static: partial sums in a buffer
built into the library) against lsq_k_gemm_add_layernorm with caller-provided scratch, through the
C ABI.  Same kernels, same slab count: the results must be the same bits.  Two calls in a row, the
second smaller, so that what the first left in the shared buffer would show."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2010_13887_amd as lib
    lib.load_library()
    return lib, torch


def _case(torch, rows, d, K, td, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    mk = lambda *s, scale=1.0: (torch.randn(*s, generator=g) * scale).to(td).cuda()
    return dict(inp=mk(rows, K), W=mk(d, K, scale=0.05), bias=mk(d, scale=0.3), x=mk(rows, d, scale=2.0),
                g=(1 + 0.3 * torch.randn(d, generator=g)).to(td).cuda(), b=mk(d, scale=0.3))


def _both(lsq, torch, c):
    x_ref, x_new = c["x"].clone(), c["x"].clone()
    lsq.k_gemm_add_layernorm(c["inp"], c["W"], c["bias"], x_ref, c["g"], c["b"], 1e-5)
    lsq.k_gemm_add_layernorm_static(c["inp"], c["W"], c["bias"], x_new, c["g"], c["b"], 1e-5)
    torch.cuda.synchronize()
    return x_ref, x_new


@pytest.mark.parametrize("half", [True, False])
@pytest.mark.parametrize("first,second", [((512, 1024, 4096), (37, 1024, 1024)), ((128, 1024, 4096), (5, 512, 2048)),
                                          ((513, 1024, 1024), (64, 1024, 4096)), ((9, 72, 40), (4, 100, 16))])
def test_static_scratch_matches_caller_scratch(env, first, second, half):
    lsq, torch = env
    td = torch.float16 if half else torch.float32
    for i, (rows, d, K) in enumerate((first, second)):
        c = _case(torch, rows, d, K, td, 1000 * i + rows + d + K)
        x_ref, x_new = _both(lsq, torch, c)
        assert torch.isfinite(x_new.float()).all()
        assert not torch.equal(x_new, c["x"])                       # it did run
        assert torch.equal(x_ref.view(torch.uint8), x_new.view(torch.uint8)), (rows, d, K)


def test_static_scratch_against_the_oracle(env):
    """...and, like the entry point it mirrors, against the plain definition."""
    from oracle import lsq_oracle as O
    lsq, torch = env
    for rows, d, K in ((200, 1024, 1024), (33, 512, 2048)):
        c = _case(torch, rows, d, K, torch.float32, rows)
        x0 = c["x"].cpu().numpy().astype(np.float64)
        a = c["inp"].cpu().numpy().astype(np.float64) @ c["W"].cpu().numpy().astype(np.float64).T + c["bias"].cpu().numpy()
        ref = O.layer_norm(x0 + a, c["g"].cpu().numpy().astype(np.float64), c["b"].cpu().numpy().astype(np.float64), 1e-5)
        x = c["x"].clone()
        lsq.k_gemm_add_layernorm_static(c["inp"], c["W"], c["bias"], x, c["g"], c["b"], 1e-5)
        np.testing.assert_allclose(x.cpu().numpy(), ref, rtol=3e-5, atol=3e-5)


def test_static_scratch_refuses_what_does_not_fit(env):
    lsq, torch = env
    limit = lsq.k_gemm_add_layernorm_static_limit()
    assert limit == 16 << 20
    lib = lsq.load_library()
    rows, d, K = 4096, 2048, 64                                     # one slab of 32 MiB
    assert lib.lsq_k_gemm_add_layernorm_scratch(0, rows, d, K) > limit
    t = torch.zeros(16, device="cuda")                              # never touched: refused before any device work
    p = ctypes.c_void_p(t.data_ptr())
    rc = lib.lsq_k_gemm_add_layernorm_static(0, p, p, p, p, p, p, rows, d, K, ctypes.c_float(1e-5), None)
    assert rc == -1 and b"built-in buffer" in lib.lsq_last_error()
    torch.cuda.synchronize()
