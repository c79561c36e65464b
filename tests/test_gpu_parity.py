"""GPU parity: HIP path (through the C ABI) vs the fp64 CPU oracle, element by element.

Bars: packing / indexing bit-exact; floating point |y_gpu - y_oracle| <= 2e-3 * B[m,n]
with B the per-output L1 bound  sum_k (|a1 T1| + |a2 T2|) |x_k|.  A tighter regression
gate (1e-5 * B for fp32 output) catches indexing mistakes the loose bar would hide:
fp32 accumulation of <= 28672 exact terms plus one rounding per scale application
stays below ~K * 2^-24 * B in the worst case and ~1e-6 * B in practice.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

TOL = 2e-3
TIGHT = 1e-5
TIGHT_F16 = 2.0 ** -10      # one extra rounding to fp16: <= 2^-11 |y| <= 2^-11 B


@pytest.fixture(scope="module")
def ptq():
    import paper_2509_16989_amd as p
    return p


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def pack(ptq, lin):
    return ptq.ptqtp_pack(dev(lin["T1"]), dev(lin["T2"]), dev(lin["a1"]), dev(lin["a2"]))


def check(y_gpu, lin, x, tight=TIGHT):
    y_ref, B = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
    y = y_gpu.detach().cpu().numpy().astype(np.float64)
    assert y.shape == y_ref.shape
    err = np.abs(y - y_ref)
    assert np.all(np.isfinite(y))
    assert np.all(err <= TOL * B), f"max err/B = {(err / np.maximum(B, 1e-300)).max():.3e}"
    assert np.all(err <= tight * B), f"regression gate: max err/B = {(err / np.maximum(B, 1e-300)).max():.3e}"
    assert np.all(y[B == 0] == 0)
    return float((err / np.maximum(B, 1e-300)).max())


# ---------------------------------------------------------------- packing: bit-exact
@pytest.mark.parametrize("N,K", [(16, 128), (16, 256), (48, 384), (1000, 1024), (1024, 1024), (7, 640), (257, 4096)])
def test_pack_unpack_roundtrip(ptq, N, K):
    lin = workloads.make_linear(N, K, 50, N, K)
    # any finite fp16 scale pattern must survive, including negative, zero, subnormal
    lin["a1"][0, 0] = np.float16(-1.5)
    lin["a2"][-1, -1] = np.float16(6e-8)
    lin["a1"][N // 2, 0] = np.float16(0.0)
    packed = pack(ptq, lin)
    assert packed.numel() == ptq.ptqtp_packed_bytes(1, N, K)
    T1, T2, a1, a2 = ptq.ptqtp_unpack(packed, N, K)
    assert np.array_equal(T1.cpu().numpy(), lin["T1"])
    assert np.array_equal(T2.cpu().numpy(), lin["T2"])
    assert np.array_equal(a1.cpu().numpy().view(np.uint16), lin["a1"].view(np.uint16))
    assert np.array_equal(a2.cpu().numpy().view(np.uint16), lin["a2"].view(np.uint16))


@pytest.mark.parametrize("N,K", [(48, 384), (257, 1024)])
def test_pack_unpack_planes_not_16_byte_aligned(ptq, N, K):
    """Planes that start 2 bytes into an allocation take the byte-wise path: same blob, same planes back."""
    lin = workloads.make_linear(N, K, 53, N, K)
    ref = pack(ptq, lin)
    bufs = []
    for name in ("T1", "T2"):
        buf = torch.zeros(N * K + 16, dtype=torch.int8, device="cuda:0")
        buf[2:2 + N * K] = dev(lin[name]).reshape(-1)
        bufs.append(buf)
    views = [b[2:2 + N * K].reshape(N, K) for b in bufs]
    assert all(v.data_ptr() % 16 == 2 for v in views)
    packed = ptq.ptqtp_pack(views[0], views[1], dev(lin["a1"]), dev(lin["a2"]))
    assert torch.equal(packed, ref)
    outs = [torch.full((N * K + 16,), 7, dtype=torch.int8, device="cuda:0") for _ in range(2)]
    from paper_2509_16989_amd import binding
    st = binding.raw().ptqtp_unpack(packed.data_ptr(), 1, N, K, 128, outs[0].data_ptr() + 2, outs[1].data_ptr() + 2, None, None,
                                torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    for out, name in zip(outs, ("T1", "T2")):
        got = out.cpu().numpy()
        assert np.array_equal(got[2:2 + N * K].reshape(N, K), lin[name])
        assert np.all(got[:2] == 7) and np.all(got[2 + N * K:] == 7)            # nothing outside the planes


def test_pack_payload_matches_memory_model(ptq):
    # appendix memory model: 4.25 bits per weight at G = 128
    for N, K in [(1024, 1024), (4096, 4096), (4096, 14336)]:
        assert (ptq.ptqtp_packed_bytes(1, N, K) - 256) * 8 == oracle.model_bits(N, K, 128)


def test_pack_agrees_with_canonical_storage(ptq):
    # unpacking the device blob and packing canonically on the host gives the oracle's bytes
    lin = workloads.make_linear(64, 512, 51)
    T1, T2, _, _ = ptq.ptqtp_unpack(pack(ptq, lin), 64, 512)
    assert np.array_equal(oracle.pack_canonical(T1.cpu().numpy()), oracle.pack_canonical(lin["T1"]))
    assert np.array_equal(oracle.pack_canonical(T2.cpu().numpy()), oracle.pack_canonical(lin["T2"]))


def test_pack_flags_bad_trit(ptq):
    lin = workloads.make_linear(32, 256, 52)
    lin["T2"][5, 77] = 2
    lin["T1"][31, 255] = -128
    lin["T1"][0, 3] = 127
    with pytest.raises(ValueError):
        pack(ptq, lin)
    # the blob is still written: the offending entries as 0, their neighbours untouched
    packed = ptq.ptqtp_pack(dev(lin["T1"]), dev(lin["T2"]), dev(lin["a1"]), dev(lin["a2"]), check=False)
    T1, T2, _, _ = ptq.ptqtp_unpack(packed, 32, 256)
    want1, want2 = lin["T1"].copy(), lin["T2"].copy()
    want2[5, 77] = 0; want1[31, 255] = 0; want1[0, 3] = 0
    assert np.array_equal(T1.cpu().numpy(), want1) and np.array_equal(T2.cpu().numpy(), want2)


# ---------------------------------------------------------------- gemv, batch 1
def test_gemv_config0(ptq):
    lin, x = workloads.config0()
    y = ptq.ptqtp_gemv(pack(ptq, lin), dev(x).reshape(-1), 1024, 1024)
    worst = check(y, lin, x)
    print(f"config0 max err/B = {worst:.3e}")


@pytest.mark.parametrize("N,K", [(16, 128), (16, 256), (48, 384), (1000, 1024), (257, 4096), (7, 640),
                                  (640, 2048), (96, 14336), (2048, 8192), (64, 28672)])
def test_gemv_shapes(ptq, N, K):
    lin = workloads.make_linear(N, K, 53, N, K)
    x = workloads.make_x(1, K, 53, N, K)
    y = ptq.ptqtp_gemv(pack(ptq, lin), dev(x).reshape(-1), N, K)
    check(y, lin, x)


@pytest.mark.parametrize("waves,depth", [(1, 1), (4, 4), (8, 2), (16, 1), (3, 4), (16, 4)])
def test_gemv_item_kernel_launch_shapes(ptq, waves, depth):
    # waves per item x records in flight: all give the same layer, including K/256 < waves,
    # an odd number of groups (K = 640) and a ragged last row tile
    try:
        ptq.ptqtp_tune("stream_waves", waves)
        ptq.ptqtp_tune("stream_depth", depth)
        for N, K in [(200, 2304), (7, 640), (1000, 1024), (33, 14336)]:
            lin = workloads.make_linear(N, K, 54, N)
            x = workloads.make_x(1, K, 54, N)
            check(ptq.ptqtp_gemv(pack(ptq, lin), dev(x).reshape(-1), N, K), lin, x)
    finally:
        ptq.ptqtp_tune("stream_waves", 0)
        ptq.ptqtp_tune("stream_depth", 0)


def test_gemv_batch_matches_oracle_and_single_calls(ptq):
    # one launch over linears of different shapes, each with its own x
    shapes = [(200, 2304), (7, 640), (1024, 1024), (33, 14336), (16, 128), (528, 4096)] * 2
    lins, xs, entries, singles = [], [], [], []
    for i, (N, K) in enumerate(shapes):
        lin = workloads.make_linear(N, K, 64, i)
        x = workloads.make_x(1, K, 64, i)
        packed = pack(ptq, lin)
        xd = dev(x).reshape(-1)
        y = torch.full((1, N), float("nan"), dtype=torch.float32, device="cuda:0")
        lins.append(lin); xs.append(x)
        entries.append((packed, xd, y, N, K))
        singles.append(ptq.ptqtp_gemv(packed, xd, N, K))
    plan = ptq.ptqtp_gemv_batch_plan(entries)
    assert plan.items == sum(((N + 15) // 16 + 15) // 16 * 16 for N, _ in shapes)
    for rep in range(3):
        ptq.ptqtp_gemv_batch(plan)
    for lin, x, ent, y1 in zip(lins, xs, entries, singles):
        check(ent[2], lin, x)
        check(y1, lin, x)
    # with the launch shape pinned, the batched launch gives the bits of the single calls
    try:
        ptq.ptqtp_tune("stream_waves", 4)
        ptq.ptqtp_tune("stream_depth", 2)
        ptq.ptqtp_gemv_batch(plan)
        for ent in entries:
            assert torch.equal(ent[2], ptq.ptqtp_gemv(ent[0], ent[1], ent[3], ent[4]))
    finally:
        ptq.ptqtp_tune("stream_waves", 0)
        ptq.ptqtp_tune("stream_depth", 0)
    # fp16 outputs
    ents16 = [(e[0], e[1], torch.empty((1, e[3]), dtype=torch.float16, device="cuda:0"), e[3], e[4]) for e in entries]
    plan16 = ptq.ptqtp_gemv_batch_plan(ents16, y_dtype=ptq.PTQTP_F16)
    ptq.ptqtp_gemv_batch(plan16)
    for lin, x, ent in zip(lins, xs, ents16):
        check(ent[2], lin, x, tight=TIGHT_F16)


@pytest.mark.parametrize("M", [1, 3, 16, 20, 40, 64])
def test_gemm_batch_matches_oracle(ptq, M):
    # one launch over linears of different shapes, M tokens each
    shapes = [(200, 2304), (7, 640), (1024, 1024), (33, 14336), (16, 128), (528, 4096)]
    lins, xs, entries = [], [], []
    for i, (N, K) in enumerate(shapes):
        lin = workloads.make_linear(N, K, 66, i)
        x = workloads.make_x(M, K, 66, i, M)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        lins.append(lin); xs.append(x)
        entries.append((pack(ptq, lin), dev(x), y, N, K))
    plan = ptq.ptqtp_gemv_batch_plan(entries)
    # shared activation tile (1 or 2 row tiles per wave; scales applied after or before the matrix pipe), per-wave loads
    for kernel, rows, fold in ((-1, 0, -1), (-1, 1, -1), (-1, 2, 0), (-1, 2, 1), (-1, 4, 0), (-1, 4, 1), (-1, 8, 0), (-1, 8, 1), (0, 0, -1)):
        try:
            ptq.ptqtp_tune("batch_rows_kernel", kernel)
            ptq.ptqtp_tune("small_rows", rows)
            ptq.ptqtp_tune("small_fold", fold)
            for ent in entries:
                ent[2].fill_(float("nan"))
            for rep in range(2):
                ptq.ptqtp_gemm_batch(plan, M)
        finally:
            ptq.ptqtp_tune("batch_rows_kernel", -1)
            ptq.ptqtp_tune("small_rows", 0)
            ptq.ptqtp_tune("small_fold", -1)
        for lin, x, ent in zip(lins, xs, entries):
            check(ent[2], lin, x)
    # fp16 outputs
    ents16 = [(e[0], e[1], torch.full((M, e[3]), float("nan"), dtype=torch.float16, device="cuda:0"), e[3], e[4]) for e in entries]
    plan16 = ptq.ptqtp_gemv_batch_plan(ents16, y_dtype=ptq.PTQTP_F16)
    ptq.ptqtp_gemm_batch(plan16, M)
    for lin, x, ent in zip(lins, xs, ents16):
        check(ent[2], lin, x, tight=TIGHT_F16)


def test_batch_plans_replay_from_a_graph(ptq):
    # a captured batched launch replayed with new activations, eager launches in between: same bits as eager
    shapes = [(200, 2304), (1024, 1024), (33, 640)]
    lins = [workloads.make_linear(N, K, 67, i) for i, (N, K) in enumerate(shapes)]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for M in (1, 12):
            xs = [torch.zeros((M, K), dtype=torch.float16, device="cuda:0") for (N, K) in shapes]
            ys = [torch.zeros((M, N), dtype=torch.float32, device="cuda:0") for (N, K) in shapes]
            plan = ptq.ptqtp_gemv_batch_plan([(pack(ptq, lin), x, y, N, K) for lin, x, y, (N, K) in zip(lins, xs, ys, shapes)])
            run = (lambda: ptq.ptqtp_gemv_batch(plan)) if M == 1 else (lambda: ptq.ptqtp_gemm_batch(plan, M))
            run()
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                run()
            for rep in range(3):
                xn = [workloads.make_x(M, K, 67, rep, i) for i, (N, K) in enumerate(shapes)]
                for x, v in zip(xs, xn):
                    x.copy_(dev(v))
                for y in ys:
                    y.fill_(float("nan"))
                g.replay()
                stream.synchronize()
                replayed = [y.clone() for y in ys]
                run()
                stream.synchronize()
                for a, y, lin, v in zip(replayed, ys, lins, xn):
                    assert torch.equal(a, y)
                    check(y, lin, v)


def test_gemv_unit_vectors_exact(ptq):
    # x = e_j returns column j of W^ = a1 T1 + a2 T2; with a2/a1 in [0.1, 0.5] the sum is exact in fp32
    N, K = 80, 768
    lin = workloads.make_linear(N, K, 55)
    packed = pack(ptq, lin)
    W = oracle.reconstruct_dense(lin["T1"], lin["T2"], lin["a1"], lin["a2"])
    cols = sorted(set([0, 1, 2, 7, 8, 31, 32, 127, 128, 255, 256, 257, 511, 767] + list(range(300, 364))))
    for j in cols:
        e = np.zeros((1, K), dtype=np.float16)
        e[0, j] = 1.0
        y = ptq.ptqtp_gemv(packed, dev(e).reshape(-1), N, K).cpu().numpy().astype(np.float64)
        assert np.array_equal(y[0], W[:, j].astype(np.float32).astype(np.float64)), f"column {j}"
        assert np.array_equal(W[:, j].astype(np.float32).astype(np.float64), W[:, j])


@pytest.mark.parametrize("M", [1, 5, 16, 33])
def test_integer_exact_bitwise(ptq, M):
    # every partial sum is exactly representable, so any summation order gives the oracle's bits
    N, K = 208, 3072
    lin, x = workloads.integer_exact_case(N, K, M, 56, M)
    y_ref, _ = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
    y = ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K).cpu().numpy().astype(np.float64)
    assert np.array_equal(y, y_ref)


@pytest.mark.parametrize("M", [2, 16, 24, 48, 64])
def test_gemm_batch_integer_exact_bitwise(ptq, M):
    # the batched small-batch kernels (scales applied after or inside the matrix pipe) on inputs whose
    # partial sums are all exactly representable: the oracle's bits in any summation order
    shapes = [(208, 3072), (40, 14336), (129, 256)]
    cases, entries = [], []
    for i, (N, K) in enumerate(shapes):
        lin, x = workloads.integer_exact_case(N, K, M, 58, i)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        cases.append((lin, x)); entries.append((pack(ptq, lin), dev(x), y, N, K))
    plan = ptq.ptqtp_gemv_batch_plan(entries)
    for fold in (0, 1):
        try:
            ptq.ptqtp_tune("small_fold", fold)
            for ent in entries:
                ent[2].fill_(float("nan"))
            ptq.ptqtp_gemm_batch(plan, M)
        finally:
            ptq.ptqtp_tune("small_fold", -1)
        for (lin, x), ent in zip(cases, entries):
            y_ref, _ = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
            assert np.array_equal(ent[2].cpu().numpy().astype(np.float64), y_ref), f"fold={fold}"


@pytest.mark.parametrize("M", [33, 40, 48, 49, 64])
def test_gemm_batch_fused_matches_rounded_weight_oracle(ptq, M):
    # ptqtp_gemm_batch_fused from 33 tokens on: the layer of the weights rounded once to fp16 (tight gate), inside the
    # bar of the unfused layer, and really another arithmetic than ptqtp_gemm_batch
    shapes = [(200, 2304), (7, 640), (1024, 1024), (33, 14336), (16, 128), (528, 4096)]
    lins, xs, entries = [], [], []
    for i, (N, K) in enumerate(shapes):
        lin = workloads.make_linear(N, K, 76, i)
        x = workloads.make_x(M, K, 76, i, M)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        lins.append(lin); xs.append(x)
        entries.append((pack(ptq, lin), dev(x), y, N, K))
    plan = ptq.ptqtp_gemv_batch_plan(entries)
    ptq.ptqtp_gemm_batch(plan, M)
    plain = [ent[2].clone() for ent in entries]
    for ent in entries:
        ent[2].fill_(float("nan"))
    for rep in range(2):
        ptq.ptqtp_gemm_batch_fused(plan, M)
    differs = False
    for lin, x, ent, y_plain in zip(lins, xs, entries, plain):
        ref_f, B_f = oracle.forward_fused(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
        ref, B = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
        got = ent[2].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref_f) <= TIGHT * B_f), f"{(np.abs(got - ref_f) / np.maximum(B_f, 1e-300)).max():.3e}"
        assert np.all(np.abs(got - ref) <= TOL * B)
        assert np.all(np.abs(got - ref) <= (2.0 ** -11 + TIGHT) * B)
        differs = differs or not torch.equal(ent[2], y_plain)
    assert differs
    # fp16 outputs
    ents16 = [(e[0], e[1], torch.empty((M, e[3]), dtype=torch.float16, device="cuda:0"), e[3], e[4]) for e in entries]
    plan16 = ptq.ptqtp_gemv_batch_plan(ents16, y_dtype=ptq.PTQTP_F16)
    ptq.ptqtp_gemm_batch_fused(plan16, M)
    for lin, x, ent in zip(lins, xs, ents16):
        ref_f, B_f = oracle.forward_fused(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
        got = ent[2].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref_f) <= TIGHT_F16 * B_f + 2.0 ** -25)


def test_gemm_batch_fused_small_m_and_integer_exact(ptq):
    # up to 32 tokens the fused call is ptqtp_gemm_batch bit for bit; on inputs whose weights and partial sums are
    # exactly representable the fused arithmetic returns the oracle's bits at every M
    shapes = [(208, 3072), (40, 14336), (129, 256)]
    for M in (1, 2, 16, 17, 32, 33, 64):
        cases, entries = [], []
        for i, (N, K) in enumerate(shapes):
            lin, x = workloads.integer_exact_case(N, K, M, 77, i)
            y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
            cases.append((lin, x)); entries.append((pack(ptq, lin), dev(x), y, N, K))
        plan = ptq.ptqtp_gemv_batch_plan(entries)
        ptq.ptqtp_gemm_batch_fused(plan, M)
        for (lin, x), ent in zip(cases, entries):
            y_ref, _ = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
            assert np.array_equal(ent[2].cpu().numpy().astype(np.float64), y_ref), M
    for M in (2, 16, 32):
        ents, lins = [], []
        for i, (N, K) in enumerate([(200, 2304), (33, 640)]):
            lin = workloads.make_linear(N, K, 78, i)
            ents.append((pack(ptq, lin), dev(workloads.make_x(M, K, 78, i, M)),
                         torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0"), N, K))
        plan = ptq.ptqtp_gemv_batch_plan(ents)
        ptq.ptqtp_gemm_batch(plan, M)
        plain = [e[2].clone() for e in ents]
        ptq.ptqtp_gemm_batch_fused(plan, M)
        for e, y_plain in zip(ents, plain):
            assert torch.equal(e[2], y_plain), M
    with pytest.raises(ptq.PtqtpError):
        ptq.ptqtp_gemm_batch_fused(plan, 65)


def test_gemv_zero_bound_gives_exact_zero(ptq):
    N, K = 64, 512
    lin = workloads.make_linear(N, K, 57)
    x = workloads.make_x(1, K, 57)
    lin["T1"][3, :] = 0
    lin["T2"][3, :] = 0                     # empty row
    lin["a1"][9, :] = 0
    lin["a2"][9, :] = 0                     # zero scales
    lin["T1"][11, 128:] = 0
    lin["T2"][11, 128:] = 0
    xz = x.copy()
    xz[0, :128] = 0                          # row 11 only meets zeros
    packed = pack(ptq, lin)
    y = ptq.ptqtp_gemv(packed, dev(xz).reshape(-1), N, K)
    check(y, lin, xz)
    yn = y.cpu().numpy()
    assert yn[0, 3] == 0 and yn[0, 9] == 0 and yn[0, 11] == 0
    y0 = ptq.ptqtp_gemv(packed, dev(np.zeros((1, K), np.float16)).reshape(-1), N, K)
    assert torch.count_nonzero(y0).item() == 0


def test_gemv_general_scales_and_subnormal_x(ptq):
    N, K = 96, 1024
    lin = workloads.make_linear(N, K, 58)
    r = np.random.default_rng(58)
    lin["a1"] = (r.standard_normal((N, K // 128)) * 3).astype(np.float16)        # signed, large
    lin["a2"] = (r.standard_normal((N, K // 128)) * 1e-6).astype(np.float16)     # subnormal fp16
    x = workloads.make_x(1, K, 58)
    x[0, ::3] = (r.standard_normal(len(x[0, ::3])) * 2e-6).astype(np.float16)    # subnormal activations
    x[0, 5] = np.float16(60000.0)
    x[0, 700] = np.float16(-30000.0)
    y = ptq.ptqtp_gemv(pack(ptq, lin), dev(x).reshape(-1), N, K)
    check(y, lin, x)
    xs = (r.standard_normal((1, K)) * 3e-6).astype(np.float16)                   # all subnormal
    check(ptq.ptqtp_gemv(pack(ptq, lin), dev(xs).reshape(-1), N, K), lin, xs)


def test_gemv_fp16_output(ptq):
    lin, x = workloads.config0()
    y = ptq.ptqtp_gemv(pack(ptq, lin), dev(x).reshape(-1), 1024, 1024, y_dtype=ptq.PTQTP_F16)
    assert y.dtype == torch.float16
    check(y, lin, x, tight=TIGHT_F16)


def test_gemv_deterministic_and_in_bounds(ptq):
    N, K = 1000, 4096
    lin = workloads.make_linear(N, K, 59)
    x = dev(workloads.make_x(1, K, 59)).reshape(-1)
    packed = pack(ptq, lin)
    guard = 64
    buf = torch.full((N + 2 * guard,), float("nan"), dtype=torch.float32, device="cuda:0")
    out = buf[guard:guard + N].view(1, N)
    first = None
    for _ in range(20):
        ptq.ptqtp_gemv(packed, x, N, K, out=out)
        cur = out.clone()
        if first is None:
            first = cur
        assert torch.equal(cur.view(torch.int32), first.view(torch.int32))
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + N:]).all()
    assert not torch.isnan(out).any()


# ---------------------------------------------------------------- small batch
@pytest.mark.parametrize("M", [2, 4, 15, 16, 17, 32, 48, 64])
def test_gemm_small_batches(ptq, M):
    N, K = 528, 2048
    lin = workloads.make_linear(N, K, 60)
    x = workloads.make_x(M, K, 60, M)
    y = ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K)
    check(y, lin, x)


@pytest.mark.parametrize("N,K,M", [(1000, 1024, 4), (257, 4096, 16), (48, 384, 64), (16, 128, 3), (96, 14336, 24),
                                    (24583, 256, 16), (24700, 384, 20), (24576, 128, 32)])   # last three: 4 row tiles per item
def test_gemm_small_shapes(ptq, N, K, M):
    lin = workloads.make_linear(N, K, 61, N, K)
    x = workloads.make_x(M, K, 61, N, M)
    check(ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K), lin, x)


@pytest.mark.parametrize("ahead", [0, 1])
@pytest.mark.parametrize("rows,waves", [(1, 1), (1, 8), (2, 2), (2, 4), (2, 8), (4, 1), (4, 4), (4, 8)])
def test_gemm_small_launch_shapes(ptq, rows, waves, ahead):
    # every (row tiles per item, waves per item) of both small-batch item kernels (ahead: loads one step ahead of the
    # arithmetic, from 17 tokens and up to two row tiles per item; elsewhere the setting falls back to the other kernel)
    try:
        ptq.ptqtp_tune("small_rows", rows)
        ptq.ptqtp_tune("small_waves", waves)
        ptq.ptqtp_tune("small_ahead", ahead)
        for N, K, M in [(200, 2304, 9), (1000, 640, 33), (48, 4096, 64), (8200, 256, 5), (1000, 640, 20), (130, 896, 47)]:
            lin = workloads.make_linear(N, K, 65, N)
            x = workloads.make_x(M, K, 65, N)
            y = ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K)
            check(y, lin, x)
            y16 = ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K, y_dtype=ptq.PTQTP_F16)
            check(y16, lin, x, tight=TIGHT_F16)
    finally:
        ptq.ptqtp_tune("small_rows", 0)
        ptq.ptqtp_tune("small_waves", 0)
        ptq.ptqtp_tune("small_ahead", -1)


# ---------------------------------------------------------------- MFMA tile (large batch / prefill)
@pytest.mark.parametrize("N,K,M", [(528, 2048, 65), (528, 2048, 128), (200, 1024, 130), (1000, 640, 257),
                                    (64, 128, 300), (2048, 4096, 512), (16, 384, 70), (4096, 256, 96)])
def test_gemm_tile_shapes(ptq, N, K, M):
    lin = workloads.make_linear(N, K, 70, N, K)
    x = workloads.make_x(M, K, 70, N, M)
    y = ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K)
    check(y, lin, x, tight=3e-5)


@pytest.mark.parametrize("N,K,M", [(528, 2048, 300), (200, 1024, 257), (1000, 640, 513), (16, 384, 256), (4096, 256, 400)])
def test_gemm_tile_variants(ptq, N, K, M):
    lin = workloads.make_linear(N, K, 73, N, K)
    x = workloads.make_x(M, K, 73, N, M)
    packed = pack(ptq, lin)
    ys = []
    for variant in (1, 2, 3, 4, 5, 0):             # 256x128, 128x128, 256x256, 128x64, 64x64 tiles, default choice
        try:
            ptq.ptqtp_tune("tile_variant", variant)
            y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
            ptq.ptqtp_gemm(packed, dev(x), N, K, out=y)
        finally:
            ptq.ptqtp_tune("tile_variant", 0)
        check(y, lin, x, tight=3e-5)
        ys.append(y)
    # every tile feeds each accumulator the same MFMA sequence: identical bits
    assert all(torch.equal(ys[0], y) for y in ys[1:])


@pytest.mark.parametrize("M", [2, 16, 33, 64])
def test_gemm_tile_forced_for_small_batches(ptq, M):
    N, K = 328, 2304
    lin = workloads.make_linear(N, K, 71)
    x = workloads.make_x(M, K, 71, M)
    try:
        ptq.ptqtp_tune("tile", 1)
        y = ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K)
        y16 = ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K, y_dtype=ptq.PTQTP_F16)
    finally:
        ptq.ptqtp_tune("tile", 0)
    check(y, lin, x, tight=3e-5)
    check(y16, lin, x, tight=TIGHT_F16)


@pytest.mark.parametrize("N,K,M", [(528, 2048, 256), (200, 1024, 300), (2048, 4096, 512), (16, 384, 257)])
def test_gemm_fused_planes_matches_rounded_weight_oracle(ptq, N, K, M):
    # PTQTP_FUSED_PLANES: the layer of the weight rounded once to fp16, exactly (tight gate), and inside the bar of the unfused layer
    lin = workloads.make_linear(N, K, 73, N, K)
    x = workloads.make_x(M, K, 73, N, M)
    ref_f, B_f = oracle.forward_fused(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    ref, B = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
    for variant in (0, 1, 2, 3, 4, 5):             # default choice, then every tile
        try:
            ptq.ptqtp_tune("tile_variant", variant)
            y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
            ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K, y_dtype=ptq.PTQTP_F32 | ptq.PTQTP_FUSED_PLANES, out=y)
        finally:
            ptq.ptqtp_tune("tile_variant", 0)
        got = y.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref_f) <= TIGHT * B_f), f"{(np.abs(got - ref_f) / B_f).max():.3e}"
        assert np.all(np.abs(got - ref) <= TOL * B)
        assert np.all(np.abs(got - ref) <= (2.0 ** -11 + TIGHT) * B)
    # the flag really selects another arithmetic
    y_plain = ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K)
    assert not torch.equal(y, y_plain)


def test_gemm_fused_planes_integer_exact_and_small_m(ptq):
    N, K, M = 272, 1024, 384
    lin, x = workloads.integer_exact_case(N, K, M, 74)
    y_ref, _ = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
    packed = pack(ptq, lin)
    y = ptq.ptqtp_gemm(packed, dev(x), N, K, y_dtype=ptq.PTQTP_F32 | ptq.PTQTP_FUSED_PLANES)
    assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref)
    y16 = ptq.ptqtp_gemm(packed, dev(x), N, K, y_dtype=ptq.PTQTP_F16 | ptq.PTQTP_FUSED_PLANES)
    assert y16.dtype == torch.float16 and np.array_equal(y16.cpu().numpy().astype(np.float64), y_ref.astype(np.float16).astype(np.float64))
    # below 256 tokens the flag has no effect: same bits as without it
    lin2 = workloads.make_linear(200, 640, 75)
    x2 = workloads.make_x(40, 640, 75)
    p2 = pack(ptq, lin2)
    assert torch.equal(ptq.ptqtp_gemm(p2, dev(x2), 200, 640, y_dtype=ptq.PTQTP_FUSED_PLANES), ptq.ptqtp_gemm(p2, dev(x2), 200, 640))
    # the other entry points do not take it
    with pytest.raises(ptq.PtqtpError):
        ptq.ptqtp_gemm_small(p2, dev(x2), 200, 640, y_dtype=ptq.PTQTP_FUSED_PLANES)


def test_gemm_tile_integer_exact_and_general_scales(ptq):
    N, K, M = 272, 1536, 144
    lin, x = workloads.integer_exact_case(N, K, M, 72)
    y_ref, _ = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
    y = ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K).cpu().numpy().astype(np.float64)
    assert np.array_equal(y, y_ref)
    r = np.random.default_rng(72)
    lin = workloads.make_linear(N, K, 72, 1)
    lin["a1"] = (r.standard_normal((N, K // 128)) * 3).astype(np.float16)
    lin["a2"] = (r.standard_normal((N, K // 128)) * 1e-6).astype(np.float16)     # subnormal fp16 scales
    x = workloads.make_x(M, K, 72, 1)
    x[:, ::5] = (r.standard_normal(x[:, ::5].shape) * 2e-6).astype(np.float16)   # subnormal activations
    check(ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K), lin, x, tight=3e-5)


@pytest.mark.parametrize("name,flag,M", [("k", 0, 2048), ("q", 0, 2048), ("q", 16, 2048), ("q", 0, 8192), ("down", 16, 4096),
                                         ("gate", 0, 2048), ("down", 0, 2048)])
def test_gemm_tile_prefill_70b_sampled(ptq, name, flag, M):
    # prefill M = 2048 .. 8192 on 70B-shaped projections (k: 1024 rows, a small tile; q: 8192 rows, the 256 x 256 tile,
    # also with fused planes; gate and down at 2048 tokens: the launches of the benchmark line, gate as 256 x 256
    # tiles for the first row blocks and a smaller tile for the rest); sampled rows and tokens against the oracle
    lin = workloads.linear_70b(name)
    N, K = lin["N"], lin["K"]
    x = workloads.x_for(name, M, K, config=4)
    y = ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K, y_dtype=flag)
    rows = np.unique(np.concatenate([[0, 15, N - 1, N - 16, N - 257], np.random.default_rng(4).integers(0, N, 48)]))
    toks = np.unique(np.concatenate([[0, 1, 63, 64, 127, 128, 255, 256, 2047, M - 1], np.random.default_rng(5).integers(0, M, 24)]))
    sub = (lin["T1"][rows], lin["T2"][rows], lin["a1"][rows], lin["a2"][rows])
    ref, B = oracle.forward(*sub, x[toks], threads=8)
    got = y.cpu().numpy().astype(np.float64)[np.ix_(toks, rows)]
    err = np.abs(got - ref)
    assert np.all(err <= TOL * B)
    if flag:
        ref_f, B_f = oracle.forward_fused(*sub, x[toks])
        assert np.all(np.abs(got - ref_f) <= 3e-5 * B_f)
    else:
        assert np.all(err <= 3e-5 * B), f"{(err / B).max():.3e}"


@pytest.mark.parametrize("flag", [0, 16])
def test_gemm_prefill_split_between_tile_sizes(ptq, flag):
    # 36 row blocks x 8 token blocks = 288 tiles of 256 x 256: the first 256 go to that tile, the last four row blocks
    # (rows 8192..9215) to smaller tiles in a second launch; rows on both sides of the seam are checked
    N, K, M = 9216, 256, 2048
    lin = workloads.make_linear(N, K, 77, 1)
    x = workloads.make_x(M, K, 77, 2)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K, y_dtype=flag, out=y)
    assert bool(torch.isfinite(y).all())
    rows = np.unique(np.concatenate([[0, 255, 256, 8191, 8192, 8447, 8448, N - 1], np.random.default_rng(8).integers(0, N, 64)]))
    toks = np.unique(np.concatenate([[0, 127, 128, 255, 256, 2047], np.random.default_rng(9).integers(0, M, 32)]))
    sub = (lin["T1"][rows], lin["T2"][rows], lin["a1"][rows], lin["a2"][rows])
    got = y.cpu().numpy().astype(np.float64)[np.ix_(toks, rows)]
    if flag:
        ref, B = oracle.forward_fused(*sub, x[toks])
    else:
        ref, B = oracle.forward(*sub, x[toks], threads=8)
    assert np.all(np.abs(got - ref) <= TIGHT * B), f"{(np.abs(got - ref) / B).max():.3e}"


@pytest.mark.parametrize("name,M,flag", [("q", 256, 0), ("q", 512, 0), ("k", 256, 0), ("k", 1024, 16), ("down", 256, 0),
                                         ("down", 512, 16), ("gate", 256, 0)])
def test_gemm_short_prompt_8b_sampled(ptq, name, M, flag):
    # short prompts on 8B-shaped projections: too few 256-row tiles to fill the chip, so the default choice is one of
    # the smaller tiles; sampled rows and tokens against the oracle
    lin = workloads.linear_8b(name)
    N, K = lin["N"], lin["K"]
    x = workloads.x_for(name, M, K, config=1)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K, y_dtype=flag, out=y)
    assert bool(torch.isfinite(y).all())
    rows = np.unique(np.concatenate([[0, 63, 64, 127, 128, N - 1], np.random.default_rng(14).integers(0, N, 48)]))
    toks = np.unique(np.concatenate([[0, 63, 64, 127, 128, M - 1], np.random.default_rng(15).integers(0, M, 24)]))
    sub = (lin["T1"][rows], lin["T2"][rows], lin["a1"][rows], lin["a2"][rows])
    got = y.cpu().numpy().astype(np.float64)[np.ix_(toks, rows)]
    ref, B = oracle.forward(*sub, x[toks], threads=8)
    assert np.all(np.abs(got - ref) <= TOL * B)
    if flag:
        ref, B = oracle.forward_fused(*sub, x[toks])
    assert np.all(np.abs(got - ref) <= 3e-5 * B), f"{(np.abs(got - ref) / B).max():.3e}"


def test_gemm_maximum_tokens_sampled(ptq):
    # the largest M the entry point takes (65536 tokens), on a narrow layer; M + 1 is refused
    N, K, M = 80, 384, 65536
    lin = workloads.make_linear(N, K, 78)
    x = workloads.make_x(M, K, 78)
    packed = pack(ptq, lin)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    ptq.ptqtp_gemm(packed, dev(x), N, K, out=y)
    assert bool(torch.isfinite(y).all())
    toks = np.unique(np.concatenate([[0, 255, 256, 32767, 32768, M - 257, M - 256, M - 1], np.random.default_rng(16).integers(0, M, 200)]))
    ref, B = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x[toks], threads=8)
    got = y.cpu().numpy().astype(np.float64)[toks]
    assert np.all(np.abs(got - ref) <= TIGHT * B)
    with pytest.raises(ptq.PtqtpError):
        ptq.ptqtp_gemm(packed, torch.zeros((M + 1, K), dtype=torch.float16, device="cuda:0"), N, K)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5])
def test_gemm_tile_fp16_output_and_guard(ptq, variant):
    # ragged rows and tokens on every tile: nothing is written outside y, fp16 output rounds once
    N, K, M = 1000, 640, 300
    lin = workloads.make_linear(N, K, 79)
    x = workloads.make_x(M, K, 79)
    buf = torch.full((M * N + 512,), 7.0, dtype=torch.float16, device="cuda:0")
    out = buf[256:256 + M * N].view(M, N)
    try:
        ptq.ptqtp_tune("tile_variant", variant)
        ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K, y_dtype=ptq.PTQTP_F16, out=out)
    finally:
        ptq.ptqtp_tune("tile_variant", 0)
    check(out, lin, x, tight=TIGHT_F16)
    assert (buf[:256] == 7).all() and (buf[256 + M * N:] == 7).all()


@pytest.mark.parametrize("seed", range(32))
def test_gemm_random_shapes(ptq, seed):
    # seeded random shapes across all regimes of ptqtp_gemm (batch 1, small batch, chunks, every tile, ragged rows,
    # tokens and an odd number of groups), fp32 / fp16 output, with and without the fused-plane flag
    r = np.random.default_rng(1000 + seed)
    N = int(r.integers(1, 1200))
    K = 128 * int(r.integers(1, 21))
    M = int(r.choice([1, int(r.integers(2, 17)), int(r.integers(17, 65)), int(r.integers(65, 256)), int(r.integers(256, 600))]))
    f16 = bool(r.integers(0, 2))
    fused = bool(r.integers(0, 2))
    lin = workloads.make_linear(N, K, 91, seed)
    x = workloads.make_x(M, K, 91, seed)
    flags = (ptq.PTQTP_F16 if f16 else ptq.PTQTP_F32) | (ptq.PTQTP_FUSED_PLANES if fused else 0)
    buf = torch.full((M * N + 256,), 7.0, dtype=torch.float16 if f16 else torch.float32, device="cuda:0")
    out = buf[128:128 + M * N].view(M, N)
    ptq.ptqtp_gemm(pack(ptq, lin), dev(x), N, K, y_dtype=flags, out=out)
    assert (buf[:128] == 7).all() and (buf[128 + M * N:] == 7).all()
    got = out.cpu().numpy().astype(np.float64)
    ref, B = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, threads=8)
    rounding = 2.0 ** -10 * B if f16 else 0.0
    assert np.all(np.abs(got - ref) <= TOL * B + rounding), (N, K, M, f16, fused)
    if fused and M >= 256:
        ref, B = oracle.forward_fused(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    assert np.all(np.abs(got - ref) <= 3e-5 * B + rounding), (N, K, M, f16, fused, float((np.abs(got - ref) / np.maximum(B, 1e-300)).max()))


def test_gemm_small_rows_match_gemv(ptq):
    # each token of a batch gets the bits batch-1 would give it? not required (different
    # reduction trees are both correct) -- but both must sit inside the tight gate
    N, K = 320, 4096
    lin = workloads.make_linear(N, K, 62)
    x = workloads.make_x(16, K, 62)
    packed = pack(ptq, lin)
    yb = ptq.ptqtp_gemm_small(packed, dev(x), N, K)
    check(yb, lin, x)
    for m in (0, 7, 15):
        y1 = ptq.ptqtp_gemv(packed, dev(x[m]), N, K)
        check(y1, lin, x[m:m + 1])


def test_gemm_small_fp16_output_and_guard(ptq):
    N, K, M = 200, 1024, 7
    lin = workloads.make_linear(N, K, 63)
    x = workloads.make_x(M, K, 63)
    buf = torch.full((M * N + 128,), 7.0, dtype=torch.float16, device="cuda:0")
    out = buf[64:64 + M * N].view(M, N)
    ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K, y_dtype=ptq.PTQTP_F16, out=out)
    check(out, lin, x, tight=TIGHT_F16)
    assert (buf[:64] == 7).all() and (buf[64 + M * N:] == 7).all()


def test_check_blob_flags_what_does_not_match(ptq):
    # the compute kernels trust N and K; the header check is what stands between a wrong blob and silent garbage
    N, K = 64, 512
    lin = workloads.make_linear(N, K, 64)
    packed = pack(ptq, lin)
    assert ptq.ptqtp_check_blob(packed, N, K) == 0
    # another shape with the very same byte count (8 records either way), and a smaller one that fits inside
    assert ptq.ptqtp_packed_bytes(1, 128, 256) == packed.numel()
    assert ptq.ptqtp_check_blob(packed, 128, 256) == ptq.PTQTP_BLOB_BAD_N | ptq.PTQTP_BLOB_BAD_K
    assert ptq.ptqtp_check_blob(packed, 48, K) == ptq.PTQTP_BLOB_BAD_N
    assert ptq.ptqtp_check_blob(packed, N, 256) == ptq.PTQTP_BLOB_BAD_K
    x = dev(workloads.make_x(1, 256, 64)).reshape(-1)
    with pytest.raises(ValueError, match="header does not match"):
        ptq.ptqtp_gemv(packed, x, 128, 256)
    with pytest.raises(ValueError, match="header does not match"):
        ptq.ptqtp_unpack(packed, 128, 256)
    # corrupted header fields: magic (bytes 0..7), layout id (8..11), group (12..15)
    for offset, bit in ((0, ptq.PTQTP_BLOB_BAD_MAGIC), (5, ptq.PTQTP_BLOB_BAD_MAGIC), (8, ptq.PTQTP_BLOB_BAD_LAYOUT),
                        (12, ptq.PTQTP_BLOB_BAD_GROUP)):
        bad = packed.clone()
        bad[offset] ^= 0x40
        assert ptq.ptqtp_check_blob(bad, N, K) == bit
        with pytest.raises(ValueError, match="header does not match"):
            ptq.ptqtp_gemv(bad, dev(workloads.make_x(1, K, 64)).reshape(-1), N, K)
    # a blob that was good and is then written to is looked at again
    xk = dev(workloads.make_x(1, K, 64)).reshape(-1)
    ptq.ptqtp_gemv(packed, xk, N, K)
    packed[0] ^= 0xff
    with pytest.raises(ValueError, match="magic"):
        ptq.ptqtp_gemv(packed, xk, N, K)
    packed[0] ^= 0xff
    check(ptq.ptqtp_gemv(packed, xk, N, K), lin, workloads.make_x(1, K, 64))


# ---------------------------------------------------------------- full-size layers, sampled rows
def _sampled_rows_check(ptq, lin, x, y, rows):
    sub_ref, B = oracle.forward(lin["T1"][rows], lin["T2"][rows], lin["a1"][rows], lin["a2"][rows], x, threads=8)
    got = y.cpu().numpy().astype(np.float64)[:, rows]
    err = np.abs(got - sub_ref)
    assert np.all(err <= TOL * B) and np.all(err <= TIGHT * B), f"{(err / B).max():.3e}"


@pytest.mark.parametrize("name", ["q", "k", "gate", "down"])
def test_gemv_8b_shapes_sampled(ptq, name):
    lin = workloads.linear_8b(name)
    N, K = lin["N"], lin["K"]
    x = workloads.x_for(name, 1, K)
    packed = pack(ptq, lin)
    y = ptq.ptqtp_gemv(packed, dev(x).reshape(-1), N, K)
    rows = np.unique(np.concatenate([np.arange(0, 32), np.arange(N - 32, N),
                                     np.random.default_rng(1).integers(0, N, 448)]))
    _sampled_rows_check(ptq, lin, x, y, rows)
    # properties that hold at any size: determinism and linearity in x (2x is exact in fp16/fp32)
    y2 = ptq.ptqtp_gemv(packed, dev(x * np.float16(2)).reshape(-1), N, K)
    assert torch.equal(y2, 2 * y)
    assert torch.equal(ptq.ptqtp_gemv(packed, dev(x).reshape(-1), N, K), y)


@pytest.mark.parametrize("M", [4, 16, 64])
def test_gemm_small_8b_q_sampled(ptq, M):
    lin = workloads.linear_8b("q")
    N, K = lin["N"], lin["K"]
    x = workloads.x_for("q", M, K, config=2)
    y = ptq.ptqtp_gemm_small(pack(ptq, lin), dev(x), N, K)
    rows = np.unique(np.concatenate([np.arange(0, 16), np.arange(N - 16, N),
                                     np.random.default_rng(2).integers(0, N, 224)]))
    _sampled_rows_check(ptq, lin, x, y, rows)


@pytest.mark.parametrize("name", ["q", "k", "gate", "down"])
def test_gemv_70b_shapes_sampled(ptq, name):
    # every 70B shape at batch 1 (streamed rows) and at 32 tokens (small-batch kernel), sampled rows
    lin = workloads.linear_70b(name)
    N, K = lin["N"], lin["K"]
    packed = pack(ptq, lin)
    x = workloads.x_for(name, 1, K, config=4)
    y = ptq.ptqtp_gemv(packed, dev(x).reshape(-1), N, K)
    rows = np.unique(np.concatenate([np.arange(0, 16), np.arange(N - 16, N), np.random.default_rng(3).integers(0, N, 256)]))
    _sampled_rows_check(ptq, lin, x, y, rows)
    x32 = workloads.x_for(name, 32, K, config=4)
    y32 = ptq.ptqtp_gemm_small(packed, dev(x32), N, K)
    assert ptq.ptqtp_gemm_route(32, N, K)[0] == ptq.PTQTP_ROUTE_SMALL
    _sampled_rows_check(ptq, lin, x32, y32, rows[:96])
    y32b = ptq.ptqtp_gemm(packed, dev(x32), N, K)                 # the dispatching entry point takes the same route
    assert torch.equal(y32b, y32)
    # 48 and 64 tokens through the small-batch entry point (on q and down: the kernel with its loads one step ahead)
    for M in (48, 64):
        xm = workloads.x_for(name, M, K, config=4)
        _sampled_rows_check(ptq, lin, xm, ptq.ptqtp_gemm_small(packed, dev(xm), N, K), rows[:64])


@pytest.mark.parametrize("N,K", [(262144, 128), (16, 262144), (1, 128), (100000, 384)])
def test_extreme_aspect_ratios_sampled(ptq, N, K):
    # very tall, very wide and the smallest layer: index arithmetic at both ends (sampled rows, batch 1, 5 and 300)
    lin = workloads.make_linear(N, K, 76, N % 1000, K % 1000)
    packed = pack(ptq, lin)
    rows = np.unique(np.concatenate([np.arange(0, min(N, 17)), np.arange(max(0, N - 17), N),
                                     np.random.default_rng(6).integers(0, N, 64)]))
    for M in (1, 5, 300):
        if M * (N + K) > 40_000_000:
            continue
        x = workloads.make_x(M, K, 76, M)
        y = ptq.ptqtp_gemm(packed, dev(x), N, K)
        assert bool(torch.isfinite(y).all())
        _sampled_rows_check(ptq, lin, x, y, rows)


def test_batch_full_stack_as_benchmarked_sampled(ptq):
    # the launch bench.py times: 32 layers x 7 linears of the 8B shapes in ONE plan; sampled rows of sampled linears
    import bench
    dev0 = torch.device("cuda:0")
    blobs, xs, ys, jobs, dims, _ = bench.build_stack(ptq, torch, workloads, 32, dev0, log=False)
    for y in ys:
        y.fill_(float("nan"))
    plan = ptq.ptqtp_gemv_batch_plan([(b, x, y, n, k) for b, x, y, (n, k) in zip(blobs, xs, ys, dims)])
    ptq.ptqtp_gemv_batch(plan)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(y).all()) for y in ys)            # every output of every linear was written
    rng = np.random.default_rng(4)
    picks = [(0, "q"), (0, "down"), (7, "k"), (15, "gate"), (31, "up"), (31, "down"), (31, "v")]
    for layer, name in picks:
        i = jobs.index((layer, name))
        lin = workloads.linear_8b(name, layer)
        N = lin["N"]
        rows = np.unique(np.concatenate([np.arange(0, 16), np.arange(N - 16, N), rng.integers(0, N, 96)]))
        _sampled_rows_check(ptq, lin, xs[i].cpu().numpy()[None, :], ys[i], rows)
    # the same stack at 4, 16 and 64 tokens per linear through the batched small-batch kernels, and at 64 tokens with
    # the planes summed in fp16 before the matrix pipe: the launches bench.py times beside the headline
    for M, fused in ((4, False), (16, False), (64, False), (64, True)):
        xm = [torch.from_numpy(workloads.x_for(name, M, k, 2, layer)).to(dev0) for (layer, name), (n, k) in zip(jobs, dims)]
        ym = [torch.full((M, n), float("nan"), dtype=torch.float32, device=dev0) for (n, k) in dims]
        planm = ptq.ptqtp_gemv_batch_plan([(b, x, y, n, k) for b, x, y, (n, k) in zip(blobs, xm, ym, dims)])
        if fused:
            ptq.ptqtp_gemm_batch_fused(planm, M)
        else:
            ptq.ptqtp_gemm_batch(planm, M)
        torch.cuda.synchronize()
        assert all(bool(torch.isfinite(y).all()) for y in ym)
        for layer, name in picks[1::2]:
            i = jobs.index((layer, name))
            lin = workloads.linear_8b(name, layer)
            rows = np.unique(np.concatenate([np.arange(lin["N"] - 16, lin["N"]), rng.integers(0, lin["N"], 48)]))
            xh = xm[i].cpu().numpy()
            if not fused:
                _sampled_rows_check(ptq, lin, xh, ym[i], rows)
            else:
                ref, B = oracle.forward_fused(lin["T1"][rows], lin["T2"][rows], lin["a1"][rows], lin["a2"][rows], xh)
                err = np.abs(ym[i].cpu().numpy().astype(np.float64)[:, rows] - ref)
                assert np.all(err <= TIGHT * B), f"{(err / B).max():.3e}"
        del xm, ym, planm


def test_smoke_entry(ptq):
    import __graft_entry__
    __graft_entry__.smoke()
