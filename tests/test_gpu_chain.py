"""GPU parity for the decode chain: fused epilogues (gated-MLP product, residual add, fp16
activations) and dependent stages, one launch per level, against the fp64 oracle stage by stage.

A stage is checked against the oracle evaluated on the input the GPU actually gave it (the
previous stage's fp16 output, read back), so each comparison isolates one stage.  Bars: with E
the oracle's first-order bound for the stage (the linear's L1 bound B pushed through the
epilogue), |out_gpu - out_oracle| <= 2e-3 * E + second-order term (+ 2^-11 |out| for an fp16
store), and a regression gate of 1e-5 * E in place of 2e-3 * E.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

TOL, TIGHT = 2e-3, 1e-5
HALF_ULP = 2.0 ** -11 * 1.001


@pytest.fixture(scope="module")
def ptq():
    import paper_2509_16989_amd as p
    return p


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def pack(ptq, lin):
    return ptq.ptqtp_pack(dev(lin["T1"]), dev(lin["T2"]), dev(lin["a1"]), dev(lin["a2"]))


def check_stage(out_gpu, lin, x16, epilogue, residual16):
    """out_gpu: tensor [n_out] or [M, n_out]; x16 / residual16: numpy float16 as the GPU saw them."""
    if x16.ndim == 1:
        x16 = x16[None, :]
        residual16 = None if residual16 is None else residual16[None, :]
        out_gpu = out_gpu[None, :]
    st = oracle.stage(lin, x16, epilogue, residual=residual16, threads=8)
    ref, E, E2 = st["out"], st["err"], st["err2"]
    got = out_gpu.detach().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape and np.all(np.isfinite(got))
    rounding = HALF_ULP * np.abs(ref) + 1e-7 if out_gpu.dtype == torch.float16 else 2.0 ** -23 * np.abs(ref)
    err = np.abs(got - ref)
    assert np.all(err <= TOL * E + TOL * TOL * E2 + rounding), f"bar: {(err / np.maximum(E, 1e-300)).max():.3e}"
    assert np.all(err <= TIGHT * E + rounding), f"regression gate: {((err - rounding) / np.maximum(E, 1e-300)).max():.3e}"


def run_chain(ptq, plan):
    ptq.ptqtp_chain_run(plan)
    torch.cuda.synchronize()


@pytest.mark.parametrize("N,K,epi,res,ydt", [
    (200, 640, "none", False, torch.float32), (200, 640, "none", True, torch.float16), (1024, 1024, "none", True, torch.float32),
    (64, 128, "swiglu", False, torch.float16), (960, 384, "swiglu", False, torch.float32), (2048, 1024, "swiglu", True, torch.float16),
    (33, 4096, "none", False, torch.float16),
])
def test_chain_single_stage(ptq, N, K, epi, res, ydt):
    lin = workloads.make_linear(N, K, 80, N, K)
    x = workloads.make_x(1, K, 80, N)[0]
    n_out = N // 2 if epi == "swiglu" else N
    r = workloads.make_x(1, n_out, 80, N, 7)[0] if res else None
    y = torch.full((n_out,), float("nan"), dtype=ydt, device="cuda:0")
    plan = ptq.ptqtp_chain_plan([dict(packed=pack(ptq, lin), x=dev(x), y=y, N=N, K=K, level=0,
                                      residual=dev(r) if res else None,
                                      epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE)])
    run_chain(ptq, plan)
    check_stage(y, lin, x, epi, r)


def build_stack(ptq, layers, H, KV, I, seed):
    """layers x {qkv -> o (+residual) -> gate_up (gated product) -> down (+residual)}; the attention
    between qkv and o is not part of the path: o reads the first H entries of qkv's output."""
    lins, stages, bufs = [], [], {}
    bufs["x0"] = torch.zeros(H, dtype=torch.float16, device="cuda:0")
    cur = bufs["x0"]
    level = 0
    for l in range(layers):
        qkv = workloads.make_linear(H + 2 * KV, H, seed, l, 1)
        o = workloads.make_linear(H, H, seed, l, 2)
        gu = workloads.make_linear(2 * I, H, seed, l, 3)
        dn = workloads.make_linear(H, I, seed, l, 4)
        t_qkv = torch.zeros(H + 2 * KV, dtype=torch.float16, device="cuda:0")
        t_attn = torch.zeros(H, dtype=torch.float16, device="cuda:0")
        t_h = torch.zeros(I, dtype=torch.float16, device="cuda:0")
        t_out = torch.zeros(H, dtype=torch.float16, device="cuda:0")
        specs = [(qkv, cur, t_qkv, None, "none"), (o, t_qkv, t_attn, cur, "none"),
                 (gu, t_attn, t_h, None, "swiglu"), (dn, t_h, t_out, t_attn, "none")]
        for lin, xin, yout, res, epi in specs:
            stages.append(dict(packed=pack(ptq, lin), x=xin, y=yout, N=lin["N"], K=lin["K"], level=level, residual=res,
                               epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE))
            lins.append((lin, xin, yout, res, epi))
            level += 1
        cur = t_out
    return lins, stages, bufs


def test_chain_dependent_stack(ptq):
    H, KV, I, layers = 384, 128, 640, 3
    lins, stages, bufs = build_stack(ptq, layers, H, KV, I, 81)
    plan = ptq.ptqtp_chain_plan(stages)
    # several runs with different inputs: a stage that read a stale copy of its input would show
    for rep in range(3):
        x0 = workloads.make_x(1, H, 81, 100 + rep)[0]
        bufs["x0"].copy_(dev(x0))
        run_chain(ptq, plan)
        for lin, xin, yout, res, epi in lins:
            k = lin["K"]
            x16 = xin.cpu().numpy()[:k]
            r16 = None if res is None else res.cpu().numpy()
            check_stage(yout, lin, x16, epi, r16)
        # the last layer's output is not the residual passed through: the chain did something
        assert not torch.equal(lins[-1][2], lins[-1][3])


def test_chain_replays_from_a_graph(ptq):
    # a decode step captured once and replayed with new inputs, eager work in between
    H, KV, I, layers = 256, 128, 384, 2
    lins, stages, bufs = build_stack(ptq, layers, H, KV, I, 82)
    plan = ptq.ptqtp_chain_plan(stages)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ptq.ptqtp_chain_run(plan)
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            ptq.ptqtp_chain_run(plan)
        for rep in range(3):
            bufs["x0"].copy_(dev(workloads.make_x(1, H, 82, 5 + rep)[0]))
            for lin, xin, yout, res, epi in lins:
                yout.zero_()
            g.replay()
            stream.synchronize()
            replayed = [t[2].clone() for t in lins]
            ptq.ptqtp_chain_run(plan)
            stream.synchronize()
            for a, t in zip(replayed, lins):
                assert torch.equal(a, t[2])
            for lin, xin, yout, res, epi in lins:
                check_stage(yout, lin, xin.cpu().numpy()[:lin["K"]], epi, None if res is None else res.cpu().numpy())


def test_chain_independent_stages_share_a_level(ptq):
    # q, k, v as three stages of one level, then o on the next
    H = 256
    x = workloads.make_x(1, H, 83, 1)[0]
    xd = dev(x)
    parts = [workloads.make_linear(n, H, 83, i) for i, n in enumerate((256, 64, 48))]
    outs = [torch.zeros(p["N"], dtype=torch.float16, device="cuda:0") for p in parts]
    o = workloads.make_linear(H, H, 83, 9)
    yo = torch.zeros(H, dtype=torch.float32, device="cuda:0")
    stages = [dict(packed=pack(ptq, p), x=xd, y=y, N=p["N"], K=H, level=0) for p, y in zip(parts, outs)]
    stages.append(dict(packed=pack(ptq, o), x=outs[0], y=yo, N=H, K=H, level=1, residual=xd))
    plan = ptq.ptqtp_chain_plan(stages)
    run_chain(ptq, plan)
    for p, y in zip(parts, outs):
        check_stage(y, p, x, "none", None)
    check_stage(yo, o, outs[0].cpu().numpy(), "none", x)


# ---------------------------------------------------------------- the chain at several tokens per stage
@pytest.mark.parametrize("M", [1, 3, 16, 24, 40, 64])
@pytest.mark.parametrize("N,K,epi,res,ydt", [
    (200, 640, "none", True, torch.float16), (1024, 1024, "none", False, torch.float32),
    (960, 384, "swiglu", False, torch.float16), (2048, 1024, "swiglu", True, torch.float32), (64, 128, "swiglu", True, torch.float16),
])
def test_chain_batch_single_stage(ptq, M, N, K, epi, res, ydt):
    lin = workloads.make_linear(N, K, 85, N, K)
    x = workloads.make_x(M, K, 85, N, M)
    n_out = N // 2 if epi == "swiglu" else N
    r = workloads.make_x(M, n_out, 85, N, M, 7) if res else None
    y = torch.full((M, n_out), float("nan"), dtype=ydt, device="cuda:0")
    plan = ptq.ptqtp_chain_plan([dict(packed=pack(ptq, lin), x=dev(x), y=y, N=N, K=K, level=0,
                                      residual=dev(r) if res else None,
                                      epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE)])
    ptq.ptqtp_chain_run_batch(plan, M)
    torch.cuda.synchronize()
    check_stage(y, lin, x, epi, r)


def build_stack_batch(ptq, layers, H, KV, I, M, seed):
    lins, stages, bufs = [], [], {}
    z = lambda n: torch.zeros((M, n), dtype=torch.float16, device="cuda:0")
    bufs["x0"] = z(H)
    cur, level = bufs["x0"], 0
    for l in range(layers):
        # o reads a buffer of its own that the test fills from qkv's output (the q part of every token)
        qkv = workloads.make_linear(H + 2 * KV, H, seed, l, 1)
        o = workloads.make_linear(H, H, seed, l, 2)
        gu = workloads.make_linear(2 * I, H, seed, l, 3)
        dn = workloads.make_linear(H, I, seed, l, 4)
        t_qkv, t_q, t_attn, t_h, t_out = z(H + 2 * KV), z(H), z(H), z(I), z(H)
        for lin, xin, yout, res, epi in [(qkv, cur, t_qkv, None, "none"), (o, t_q, t_attn, cur, "none"),
                                         (gu, t_attn, t_h, None, "swiglu"), (dn, t_h, t_out, t_attn, "none")]:
            stages.append(dict(packed=pack(ptq, lin), x=xin, y=yout, N=lin["N"], K=lin["K"], level=level, residual=res,
                               epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE))
            lins.append((lin, xin, yout, res, epi))
            level += 1
        bufs[("q", l)] = (t_qkv, t_q)
        cur = t_out
    return lins, stages, bufs


@pytest.mark.parametrize("M", [65, 130, 256, 300])
@pytest.mark.parametrize("N,K,epi,res,ydt", [
    (200, 640, "none", True, torch.float16), (1024, 1024, "none", False, torch.float32),
    (960, 384, "swiglu", False, torch.float16), (2048, 1024, "swiglu", True, torch.float32), (64, 128, "swiglu", True, torch.float16),
    (8192, 256, "swiglu", True, torch.float16), (9216, 256, "none", True, torch.float16),
])
def test_chain_batch_single_stage_on_tiles(ptq, M, N, K, epi, res, ydt):
    # more than 64 tokens: an MFMA tile with the epilogue in its store (a gated stage pairs gate and up tiles per wave)
    lin = workloads.make_linear(N, K, 87, N, K)
    x = workloads.make_x(M, K, 87, N, M)
    n_out = N // 2 if epi == "swiglu" else N
    r = workloads.make_x(M, n_out, 87, N, M, 7) if res else None
    y = torch.full((M, n_out), float("nan"), dtype=ydt, device="cuda:0")
    plan = ptq.ptqtp_chain_plan([dict(packed=pack(ptq, lin), x=dev(x), y=y, N=N, K=K, level=0,
                                      residual=dev(r) if res else None,
                                      epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE)])
    ptq.ptqtp_chain_run_batch(plan, M)
    torch.cuda.synchronize()
    check_stage(y, lin, x, epi, r)


@pytest.mark.parametrize("N,K,M,epi", [(1024, 1024, 256, "none"), (2048, 512, 300, "swiglu")])
def test_chain_batch_fused_planes_stage(ptq, N, K, M, epi):
    # a stage with the fused-plane flag: the stage of the weight rounded once to fp16 (w16 = fp16(a1 t1 + a2 t2))
    lin = workloads.make_linear(N, K, 89, N)
    x = workloads.make_x(M, K, 89, N)
    n_out = N // 2 if epi == "swiglu" else N
    r = workloads.make_x(M, n_out, 89, 7)
    y = torch.full((M, n_out), float("nan"), dtype=torch.float32, device="cuda:0")
    y_plain = torch.empty_like(y)
    mk = lambda out, fused: ptq.ptqtp_chain_plan([dict(packed=pack(ptq, lin), x=dev(x), y=out, N=N, K=K, level=0, residual=dev(r), fused_planes=fused,
                                                       epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE)])
    ptq.ptqtp_chain_run_batch(mk(y, True), M)
    ptq.ptqtp_chain_run_batch(mk(y_plain, False), M)
    torch.cuda.synchronize()
    check_stage(y_plain, lin, x, epi, r)
    assert not torch.equal(y, y_plain)
    # the rounded-weight layer, exactly: rebuild it as a one-plane layer with unit scales is not possible (w16 is not a
    # trit), so compare through the oracle's fused forward and redo the epilogue in float64
    yf, Bf = oracle.forward_fused(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    if epi == "swiglu":
        I = N // 2
        ref = oracle.swiglu(yf, I)
        E = oracle.SILU_LIPSCHITZ * Bf[:, :I] * np.abs(yf[:, I:]) + np.abs(yf[:, :I]) * Bf[:, I:] + oracle.SILU_LIPSCHITZ * Bf[:, :I] * Bf[:, I:]
    else:
        ref, E = yf, Bf
    ref = ref + r.astype(np.float64)
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 1e-5 * E + 2.0 ** -23 * np.abs(ref))


@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("epi", ["none", "swiglu"])
def test_chain_batch_every_tile_with_epilogue(ptq, variant, epi):
    # each tile kind with the epilogue in its store, ragged rows and tokens (a gated stage cannot use the 64 x 64 tile,
    # whose waves own one row tile: the override is ignored there)
    N, K, M = 1184, 640, 290
    lin = workloads.make_linear(N, K, 90, N)
    x = workloads.make_x(M, K, 90, N)
    n_out = N // 2 if epi == "swiglu" else N
    r = workloads.make_x(M, n_out, 90, 7)
    y = torch.full((M, n_out), float("nan"), dtype=torch.float16, device="cuda:0")
    plan = ptq.ptqtp_chain_plan([dict(packed=pack(ptq, lin), x=dev(x), y=y, N=N, K=K, level=0, residual=dev(r),
                                      epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE)])
    try:
        ptq.ptqtp_tune("tile_variant", variant)
        ptq.ptqtp_chain_run_batch(plan, M)
        torch.cuda.synchronize()
    finally:
        ptq.ptqtp_tune("tile_variant", 0)
    check_stage(y, lin, x, epi, r)


def test_chain_batch_in_place_residual_on_tiles(ptq):
    # y may be the stage's own residual buffer (the residual stream updated in place)
    N, K, M = 512, 384, 200
    lin = workloads.make_linear(N, K, 88)
    x = workloads.make_x(M, K, 88)
    r = workloads.make_x(M, N, 88, 7)
    buf = dev(r).clone()
    plan = ptq.ptqtp_chain_plan([dict(packed=pack(ptq, lin), x=dev(x), y=buf, N=N, K=K, level=0, residual=buf)])
    ptq.ptqtp_chain_run_batch(plan, M)
    torch.cuda.synchronize()
    check_stage(buf, lin, x, "none", r)


@pytest.mark.parametrize("M", [5, 33, 150])
def test_chain_batch_dependent_stack(ptq, M):
    # with M tokens a row of qkv's output is not contiguous with the next token's q part, so o gets its input through
    # a copy the test makes between two runs of sub-chains (stands in for attention); every stage is checked on its real input
    H, KV, I, layers = 256, 128, 384, 2
    lins, stages, bufs = build_stack_batch(ptq, layers, H, KV, I, M, 86)
    bufs["x0"].copy_(dev(workloads.make_x(M, H, 86, M)))
    for l in range(layers):
        first = ptq.ptqtp_chain_plan(stages[4 * l: 4 * l + 1])
        rest = ptq.ptqtp_chain_plan(stages[4 * l + 1: 4 * l + 4])
        ptq.ptqtp_chain_run_batch(first, M)
        t_qkv, t_q = bufs[("q", l)]
        t_q.copy_(t_qkv[:, :H])
        ptq.ptqtp_chain_run_batch(rest, M)
    torch.cuda.synchronize()
    for lin, xin, yout, res, epi in lins:
        check_stage(yout, lin, xin.cpu().numpy(), epi, None if res is None else res.cpu().numpy())
    assert not torch.equal(lins[-1][2], lins[-1][3])


# ---------------------------------------------------------------- every launch shape of the batch-1 chain kernel
@pytest.mark.parametrize("depth", [1, 2, 4])
@pytest.mark.parametrize("waves", [2, 4, 8, 16])
def test_chain_forced_launch_shapes(ptq, waves, depth):
    # waves per item x records in flight per wave, forced through the tuning hook, on plain and gated stages:
    # an odd number of groups (K = 640: the last record is half padding), a ragged last row tile (N = 200),
    # rows long enough for several rounds of the K loop (K = 4224), fp16 and fp32 stores, with and without residual
    cases = [(200, 640, "none", True, torch.float16), (200, 640, "none", False, torch.float32),
             (40, 4224, "none", True, torch.float32), (960, 640, "swiglu", False, torch.float16),
             (64, 4224, "swiglu", True, torch.float32), (2048, 1024, "swiglu", True, torch.float16)]
    try:
        ptq.ptqtp_tune("chain_waves", waves)
        ptq.ptqtp_tune("chain_depth", depth)
        for N, K, epi, res, ydt in cases:
            lin = workloads.make_linear(N, K, 91, N, K)
            x = workloads.make_x(1, K, 91, N)[0]
            n_out = N // 2 if epi == "swiglu" else N
            r = workloads.make_x(1, n_out, 91, N, 7)[0] if res else None
            y = torch.full((n_out,), float("nan"), dtype=ydt, device="cuda:0")
            plan = ptq.ptqtp_chain_plan([dict(packed=pack(ptq, lin), x=dev(x), y=y, N=N, K=K, level=0,
                                              residual=dev(r) if res else None,
                                              epilogue=ptq.PTQTP_EPI_SWIGLU if epi == "swiglu" else ptq.PTQTP_EPI_NONE)])
            run_chain(ptq, plan)
            check_stage(y, lin, x, epi, r)
    finally:
        ptq.ptqtp_tune("chain_waves", 0)
        ptq.ptqtp_tune("chain_depth", 0)


def test_chain_forced_launch_shapes_agree_bitwise_on_integer_inputs(ptq):
    # integer-exact inputs: every launch shape must give the same bits (any summation order is exact)
    N, K = 96, 2304
    lin, x = workloads.integer_exact_case(N, K, 1, 92)
    blob, xd = pack(ptq, lin), dev(x[0])
    outs = []
    try:
        for waves in (2, 4, 8, 16):
            for depth in (1, 2, 4):
                ptq.ptqtp_tune("chain_waves", waves)
                ptq.ptqtp_tune("chain_depth", depth)
                y = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda:0")
                run_chain(ptq, ptq.ptqtp_chain_plan([dict(packed=blob, x=xd, y=y, N=N, K=K, level=0)]))
                outs.append(y)
    finally:
        ptq.ptqtp_tune("chain_waves", 0)
        ptq.ptqtp_tune("chain_depth", 0)
    ref, _ = oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    for y in outs:
        assert np.array_equal(y.cpu().numpy().astype(np.float64), ref[0])


# ---------------------------------------------------------------- the 8B chain exactly as bench.py times it
def _fused_host_linear(names, layer, scale=None):
    """Host copy of what bench.build_decode_chain packs for one stage: the named linears' rows stacked, the
    scales multiplied by `scale` in binary16 (one rounding, as the device multiply does)."""
    parts = [workloads.linear_8b(nm, layer) for nm in names]
    lin = {k: np.concatenate([p[k] for p in parts]) for k in ("T1", "T2", "a1", "a2")}
    if scale is not None:
        lin["a1"] = (lin["a1"] * np.float16(scale)).astype(np.float16)
        lin["a2"] = (lin["a2"] * np.float16(scale)).astype(np.float16)
    lin["N"], lin["K"] = lin["T1"].shape
    return lin


def test_chain_full_8b_stack_as_benchmarked_sampled(ptq):
    # the dependent decode step bench.py reports: 32 layers x {qkv, o, gate|up, down} at the 8B shapes, built by the
    # benchmark's own builder, run eagerly and replayed from a hipGraph as it is timed.  Layers 0 and 31: every stage
    # on sampled rows against the oracle fed the fp16 input the GPU gave that stage; all layers: outputs finite and
    # the replay bit-identical to the eager run.
    import bench
    dev0 = torch.device("cuda:0")
    blobs, xs, ys, jobs, dims, _ = bench.build_stack(ptq, torch, workloads, 32, dev0, log=False)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        stages, x0, _ = bench.build_decode_chain(ptq, torch, blobs, jobs, dims)
        del blobs, xs, ys
        assert len(stages) == 128
        plan = ptq.ptqtp_chain_plan(stages)
        for st in stages:
            st["y"].fill_(float("nan"))
        ptq.ptqtp_chain_run(plan)
        stream.synchronize()
        eager = [st["y"].clone() for st in stages]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            ptq.ptqtp_chain_run(plan)
        for st in stages:
            st["y"].fill_(float("nan"))
        g.replay()
        stream.synchronize()
    for st, e in zip(stages, eager):
        assert bool(torch.isfinite(st["y"].float()).all())
        assert torch.equal(st["y"], e)
    rng = np.random.default_rng(8)
    spec = [(("q", "k", "v"), None, "none"), (("o",), bench.CHAIN_O_SCALE, "none"),
            (("gate", "up"), None, "swiglu"), (("down",), bench.CHAIN_DOWN_SCALE, "none")]
    for layer in (0, 31):
        for s, (names, scale, epi) in enumerate(spec):
            st = stages[4 * layer + s]
            lin = _fused_host_linear(names, layer, scale)
            N, K = lin["N"], lin["K"]
            assert (N, K) == (st["N"], st["K"])
            # the packed stage holds exactly these planes and scales (bit-exact, whole matrix)
            t1, t2, s1, s2 = ptq.ptqtp_unpack(st["packed"], N, K)
            assert np.array_equal(t1.cpu().numpy(), lin["T1"]) and np.array_equal(t2.cpu().numpy(), lin["T2"])
            assert np.array_equal(s1.cpu().numpy().view(np.uint16), lin["a1"].view(np.uint16))
            assert np.array_equal(s2.cpu().numpy().view(np.uint16), lin["a2"].view(np.uint16))
            del t1, t2, s1, s2
            n_out = N // 2 if epi == "swiglu" else N
            rows = np.unique(np.concatenate([np.arange(0, 16), np.arange(n_out - 16, n_out), rng.integers(0, n_out, 256)]))
            sel = np.concatenate([rows, n_out + rows]) if epi == "swiglu" else rows
            sub = {k: lin[k][sel] for k in ("T1", "T2", "a1", "a2")}
            sub["N"], sub["K"] = len(sel), K
            x16 = st["x"].cpu().numpy()[:K]
            r16 = None if st["residual"] is None else st["residual"].cpu().numpy()[rows]
            check_stage(st["y"][torch.from_numpy(rows).to(dev0)], sub, x16, epi, r16)


def test_chain_wide_level_and_table_lookup(ptq):
    # a level of six independent stages (more than travel as kernel arguments: the items find their stage through the
    # device-side plan), followed by a dependent level of two; then the same chain with every level forced through
    # the plan table -- bit-identical, and both against the oracle
    H = 256
    x = workloads.make_x(1, H, 93, 1)[0]
    xd = dev(x)
    sizes = (64, 48, 256, 16, 100, 32)
    parts = [workloads.make_linear(n, H, 93, i) for i, n in enumerate(sizes)]
    outs = [torch.full((p["N"],), float("nan"), dtype=torch.float16, device="cuda:0") for p in parts]
    o = workloads.make_linear(H, H, 93, 9)
    g = workloads.make_linear(128, H, 93, 10)
    yo = torch.full((H,), float("nan"), dtype=torch.float32, device="cuda:0")
    yg = torch.full((64,), float("nan"), dtype=torch.float16, device="cuda:0")
    stages = [dict(packed=pack(ptq, p), x=xd, y=y, N=p["N"], K=H, level=0) for p, y in zip(parts, outs)]
    stages.append(dict(packed=pack(ptq, o), x=outs[2], y=yo, N=H, K=H, level=1, residual=xd))
    stages.append(dict(packed=pack(ptq, g), x=outs[2], y=yg, N=128, K=H, level=1, epilogue=ptq.PTQTP_EPI_SWIGLU))
    plan = ptq.ptqtp_chain_plan(stages)
    run_chain(ptq, plan)
    first = [t.clone() for t in outs + [yo, yg]]
    for p, y in zip(parts, outs):
        check_stage(y, p, x, "none", None)
    check_stage(yo, o, outs[2].cpu().numpy(), "none", x)
    check_stage(yg, g, outs[2].cpu().numpy(), "swiglu", None)
    for t in outs + [yo, yg]:
        t.fill_(float("nan"))
    try:
        ptq.ptqtp_tune("chain_table", 1)
        run_chain(ptq, plan)
    finally:
        ptq.ptqtp_tune("chain_table", 0)
    for a, b in zip(first, outs + [yo, yg]):
        assert torch.equal(a, b)
