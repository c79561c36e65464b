"""GPU parity for the quantizer: ptqtp_quantize (C ABI) vs the binary64 oracle.  Trits, stored scales and
iteration counts are integers / bit patterns: the bar is bit-exact.  (The stopping rule compares a
binary64 norm with eps; the two sides add the same terms in different orders, so the iteration count
could only differ if the norm landed within ~1e-13 relative of eps.)"""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ptq():
    import paper_2509_16989_amd as p
    return p


def _weights(n, k, seed, scale=0.02):
    return (np.random.default_rng([16989, 77, seed]).standard_normal((n, k)) * scale).astype(np.float16)


def _run(ptq, W, **kw):
    T1, T2, a1, a2, it = ptq.ptqtp_quantize(torch.from_numpy(W).to("cuda:0"), **kw)
    torch.cuda.synchronize()
    return (T1.cpu().numpy(), T2.cpu().numpy(), a1.cpu().numpy(), a2.cpu().numpy(), int(it.item()))


def _same(got, ref):
    T1, T2, a1, a2, it = got
    assert it == ref["iters"]
    assert np.array_equal(T1, ref["T1"]), f"{(T1 != ref['T1']).sum()} trits differ in plane 1"
    assert np.array_equal(T2, ref["T2"]), f"{(T2 != ref['T2']).sum()} trits differ in plane 2"
    assert np.array_equal(a1.view(np.uint16), ref["a1"].view(np.uint16))
    assert np.array_equal(a2.view(np.uint16), ref["a2"].view(np.uint16))


@pytest.mark.parametrize("N,K", [(64, 1024), (7, 640), (200, 128), (1, 256), (33, 4096)])
def test_quantize_matches_oracle_paper_settings(ptq, N, K):
    W = _weights(N, K, N + K)
    _same(_run(ptq, W), oracle.quantize(W))                     # T_max = 50, eps = 1e-4


@pytest.mark.parametrize("iters", [0, 1, 2, 3, 10, 50])
def test_quantize_fixed_iteration_counts(ptq, iters):
    W = _weights(48, 512, iters)
    _same(_run(ptq, W, max_iters=iters, eps=0.0), oracle.quantize(W, max_iters=iters, eps=0.0))


@pytest.mark.parametrize("eps", [1e-2, 1e-3, 1e-5])
def test_quantize_stopping_rule(ptq, eps):
    W = _weights(40, 768, 3)
    ref = oracle.quantize(W, eps=eps)
    got = _run(ptq, W, eps=eps)
    _same(got, ref)
    assert 1 <= got[4] <= 50


def test_quantize_special_weights(ptq):
    r = np.random.default_rng(5)
    N, K = 24, 512
    W = _weights(N, K, 9)
    W[0] = 0.0                                   # all-zero row
    W[1, :128] = -0.0
    W[2] = (r.integers(-1, 2, K) * 0.0625).astype(np.float16)          # exactly ternary
    W[3] = np.float16(0.03125)                   # constant
    W[4] = (r.standard_normal(K) * 3e-6).astype(np.float16)            # binary16 subnormals
    W[5] = (r.standard_normal(K) * 2000).astype(np.float16)            # large
    W[6, ::2] = 0.0
    W[7] = np.where(r.random(K) < 0.5, 1.0, -1.0).astype(np.float16) * np.float16(0.01)   # binary
    _same(_run(ptq, W), oracle.quantize(W))
    _same(_run(ptq, W, max_iters=4, eps=0.0), oracle.quantize(W, max_iters=4, eps=0.0))


def test_quantize_is_deterministic_and_leaves_guards(ptq):
    W = torch.from_numpy(_weights(100, 1024, 11)).to("cuda:0")
    a = ptq.ptqtp_quantize(W)
    b = ptq.ptqtp_quantize(W)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_quantize_then_pack_then_forward(ptq):
    # end to end: quantise a weight matrix, pack it, run the layer, compare with the oracle fed the oracle's
    # own decomposition -- and with the dense fp16 layer it approximates
    N, K = 256, 1024
    W = _weights(N, K, 13)
    T1, T2, a1, a2, it = ptq.ptqtp_quantize(torch.from_numpy(W).to("cuda:0"))
    packed = ptq.ptqtp_pack(T1, T2, a1, a2)
    x = workloads.make_x(4, K, 88)
    y = ptq.ptqtp_gemm_small(packed, torch.from_numpy(x).to("cuda:0"), N, K).cpu().numpy().astype(np.float64)
    ref = oracle.quantize(W)
    y_ref, B = oracle.forward(ref["T1"], ref["T2"], ref["a1"], ref["a2"], x)
    assert np.all(np.abs(y - y_ref) <= 1e-5 * B)
    y_dense = x.astype(np.float64) @ W.astype(np.float64).T
    rel = np.linalg.norm(y - y_dense) / np.linalg.norm(y_dense)
    assert rel < 0.3                                 # the decomposition carries ~17 % relative weight error


def test_quantize_8b_k_projection_sampled(ptq):
    # full-size layer (1024 x 4096): all scales, iteration count, and the trits of sampled rows
    W = _weights(1024, 4096, 17)
    got = _run(ptq, W)
    rows = np.unique(np.random.default_rng(1).integers(0, 1024, 64))
    full = oracle.quantize(W)                        # ~4 s on the host
    assert got[4] == full["iters"]
    assert np.array_equal(got[2].view(np.uint16), full["a1"].view(np.uint16))
    assert np.array_equal(got[3].view(np.uint16), full["a2"].view(np.uint16))
    assert np.array_equal(got[0][rows], full["T1"][rows]) and np.array_equal(got[1][rows], full["T2"][rows])
    assert np.array_equal(got[0], full["T1"]) and np.array_equal(got[1], full["T2"])
