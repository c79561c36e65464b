"""ptqtp_quantize_static -- the entry point that allocates nothing -- against ptqtp_quantize, through the C ABI.

Same kernels, workspace in the library's static device array instead of a caller's buffer: trits, stored scales
and iteration count must be bit-identical, on two calls in a row of which the second is smaller (the array keeps
the first call's contents), and oversized layers must be refused before anything is launched.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ptq():
    import paper_2509_16989_amd as p
    return p


def _weights(N, K, seed):
    rng = np.random.default_rng(seed)
    return torch.from_numpy((rng.standard_normal((N, K)) * 0.02).astype(np.float16)).to("cuda:0")


def _outputs(N, K):
    dev = "cuda:0"
    return (torch.full((N, K), 7, dtype=torch.int8, device=dev), torch.full((N, K), 7, dtype=torch.int8, device=dev),
            torch.full((N, K // 128), float("nan"), dtype=torch.float16, device=dev),
            torch.full((N, K // 128), float("nan"), dtype=torch.float16, device=dev),
            torch.full((1,), -1, dtype=torch.int32, device=dev))


def test_quantize_static_matches_quantize_on_two_calls_in_a_row(ptq):
    from paper_2509_16989_amd import binding
    lib = binding.raw()
    stream = torch.cuda.current_stream().cuda_stream
    for N, K, seed in ((768, 1024, 1), (200, 384, 2)):          # the second call is smaller than the first
        W = _weights(N, K, seed)
        ref = ptq.ptqtp_quantize(W)
        out = _outputs(N, K)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        st = lib.ptqtp_quantize_static(W.data_ptr(), N, K, 128, 50, 1e-4, out[0].data_ptr(), out[1].data_ptr(),
                                       out[2].data_ptr(), out[3].data_ptr(), out[4].data_ptr(), stream)
        assert st == 0
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for got, want in zip(out, ref):
            assert torch.equal(got.view(torch.uint8) if got.dtype == torch.int8 else got.view(torch.int16) if got.dtype == torch.float16 else got,
                               want.view(torch.uint8) if want.dtype == torch.int8 else want.view(torch.int16) if want.dtype == torch.float16 else want)
        assert 1 <= int(out[4].item()) <= 50
    # a fixed iteration count and the state-only call (max_iters = 0) take the same route
    W = _weights(64, 256, 3)
    for iters in (0, 3):
        ref = ptq.ptqtp_quantize(W, max_iters=iters)
        out = _outputs(64, 256)
        ptq.ptqtp_quantize_static(W, *out, max_iters=iters)
        torch.cuda.synchronize()
        for got, want in zip(out[:2], ref[:2]):
            assert torch.equal(got, want)
        assert torch.equal(out[2].view(torch.int16), ref[2].view(torch.int16))
        assert torch.equal(out[3].view(torch.int16), ref[3].view(torch.int16))
        assert int(out[4].item()) == int(ref[4].item()) == iters


def test_quantize_static_refuses_what_does_not_fit(ptq):
    from paper_2509_16989_amd import binding
    lib = binding.raw()
    # 524,288 units fit exactly; one row more does not.  Nothing is launched for a refused call: the outputs keep their fill.
    assert lib.ptqtp_quantize_workspace_bytes(16384, 4096, 128) == ptq.PTQTP_QUANTIZE_STATIC_BYTES
    N, K = 16385, 4096
    W = torch.zeros((8, K), dtype=torch.float16, device="cuda:0")       # never read: the call is refused on the host
    out = _outputs(8, K)
    st = lib.ptqtp_quantize_static(W.data_ptr(), N, K, 128, 50, 1e-4, out[0].data_ptr(), out[1].data_ptr(),
                                   out[2].data_ptr(), out[3].data_ptr(), out[4].data_ptr(), None)
    assert st == 4                                                       # PTQTP_ERR_SIZE
    torch.cuda.synchronize()
    assert bool((out[0] == 7).all()) and int(out[4].item()) == -1
    with pytest.raises(ptq.PtqtpError):
        ptq.ptqtp_quantize_static(torch.zeros((4, 100), dtype=torch.float16, device="cuda:0"), *_outputs(4, 128))
