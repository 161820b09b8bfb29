"""csgs_layer_gemm_grad_w_static, the entry point that allocates nothing (its partial sums live in a
static device buffer of the library), against csgs_layer_gemm_grad_w with a caller's scratch: same
kernels, so the same bits, and both within the stated tolerance of the oracle.  Two calls in a row,
the second with a smaller input (the buffer keeps the first call's contents)."""
import sys

import numpy as np
import pytest

import chain
import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_grad_w_without_allocation_matches_the_scratch_form():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2101_07706_amd import csgs
    csgs.lib()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    for M, K, N in [(8192, 256, 256), (1500, 100, 47)]:          # the second call is the smaller one
        print(f"[no-alloc] dW for M={M} K={K} N={N}", flush=True)
        sys.stdout.flush()
        Z = rng.standard_normal((M, K)).astype(np.float32)
        G = rng.standard_normal((M, N)).astype(np.float32)
        Zd, Gd = torch.from_numpy(Z).to(dev), torch.from_numpy(G).to(dev)
        want = torch.full((K, N), float("nan"), dtype=torch.float32, device=dev)
        got = torch.full((K, N), float("nan"), dtype=torch.float32, device=dev)
        nbytes = csgs.csgs_layer_gemm_grad_w_scratch_bytes(M, K, N)
        assert 0 < nbytes <= csgs.GRAD_W_STATIC_BYTES
        scratch = torch.empty(nbytes // 8 + 32, dtype=torch.int64, device=dev)
        csgs.csgs_layer_gemm_grad_w(Zd, Gd, want, scratch)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        csgs.csgs_layer_gemm_grad_w_static(Zd, Gd, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got, want), "static-scratch form differs from the caller-scratch form"
        chain.assert_close(got.cpu().numpy(), oracle.layer_gemm_grad_w(Z, G), chain.RTOL, chain.ATOL, "dW, static scratch")
        # with a device row count below the capacity
        m = M - 129
        cnt = torch.tensor([m], dtype=torch.int32, device=dev)
        want.fill_(float("nan"))
        got.fill_(float("nan"))
        csgs.csgs_layer_gemm_grad_w(Zd, Gd, want, scratch, M_dev=cnt)
        csgs.csgs_layer_gemm_grad_w_static(Zd, Gd, got, M_dev=cnt)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        chain.assert_close(got.cpu().numpy(), oracle.layer_gemm_grad_w(Z[:m], G[:m]), chain.RTOL, chain.ATOL, "dW, static scratch, M_dev")
    # a shape whose partial sums exceed the static buffer is rejected on the host, nothing is enqueued
    M, K, N = 65536, 2048, 2304
    assert csgs.csgs_layer_gemm_grad_w_scratch_bytes(M, K, N) > csgs.GRAD_W_STATIC_BYTES
    p = 4096   # never dereferenced: the size check comes first
    L = csgs.lib()
    import ctypes as C
    rc = L.csgs_layer_gemm_grad_w_static(C.c_void_p(p), K, C.c_void_p(p), N, M, None, K, N, C.c_void_p(p), N, None)
    assert rc == csgs.EWORKSPACE
