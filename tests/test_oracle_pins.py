"""Pins for the fp64 CPU oracle (no GPU).  Each test ties the oracle to something
other than itself: a library routine, exact rational brute force, a closed form
of the paper, or an invariant of the layer's definition (paper, Eq. 1-2 with
group-wise scales)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _small(N=48, K=512, M=3, key=7, group=128):
    lin = workloads.make_linear(N, K, 90, key, group=group)
    x = workloads.make_x(M, K, 90, key)
    return lin, x


def _fwd(lin, x, **kw):
    return oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, group=lin["group"], **kw)


# ---------------------------------------------------------------- binary16 decoder
def test_half_decoder_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)          # numpy's own converter
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_half_decoder_landmarks():
    # values fixed by IEEE 754 binary16, independent of any library
    assert oracle.half_to_double(0x3C00) == 1.0
    assert oracle.half_to_double(0xBC00) == -1.0
    assert oracle.half_to_double(0x0001) == 2.0 ** -24
    assert oracle.half_to_double(0x0400) == 2.0 ** -14
    assert oracle.half_to_double(0x7BFF) == 65504.0
    assert oracle.half_to_double(0x3555) == 0.333251953125


# ---------------------------------------------------------------- definition -> library matmul
@pytest.mark.parametrize("N,K,M,group", [(48, 512, 3, 128), (16, 256, 1, 128), (33, 384, 5, 128),
                                          (8, 64, 2, 16), (5, 1024, 4, 256)])
def test_matches_dense_reconstruction(N, K, M, group):
    lin, x = _small(N, K, M, key=N + K, group=group)
    y, B = _fwd(lin, x)
    yd = oracle.forward_dense(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, group=group)
    assert y.shape == (M, N) and yd.shape == (M, N)
    assert np.all(np.abs(y - yd) <= 1e-12 * B + 1e-300)


def test_config0_matches_dense():
    lin, x = workloads.config0()
    y, B = _fwd(lin, x)
    yd = oracle.forward_dense(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    assert np.all(np.abs(y - yd) <= 1e-12 * B)
    assert np.all(B >= np.abs(y))


# ---------------------------------------------------------------- exact brute force, hand-sized
def test_bruteforce_rational_tiny():
    # N=2, K=8, G=4, M=2 written out by hand; everything is a binary16 value,
    # so exact rational arithmetic gives the one true answer.
    T1 = np.array([[1, 0, -1, 1, 0, 0, 1, -1], [-1, -1, 0, 1, 1, 0, 0, 1]], dtype=np.int8)
    T2 = np.array([[0, 1, 1, -1, 1, 0, -1, 0], [1, 0, 0, -1, 0, -1, 1, 1]], dtype=np.int8)
    a1 = np.array([[0.5, 0.03125], [0.0999755859375, 1.5]], dtype=np.float16)
    a2 = np.array([[0.125, -0.25], [0.0, 0.0078125]], dtype=np.float16)
    x = np.array([[1.5, -2.0, 0.25, 3.0, -0.5, 4.0, 1.0, -1.25],
                  [0.1, 0.2, -0.3, 0.4, 100.0, -7.0, 0.001, 2.0]], dtype=np.float16)
    y, B = oracle.forward(T1, T2, a1, a2, x, group=4)
    for m in range(2):
        for n in range(2):
            acc = Fraction(0)
            bnd = Fraction(0)
            for k in range(8):
                g = k // 4
                w = Fraction(float(a1[n, g])) * int(T1[n, k]) + Fraction(float(a2[n, g])) * int(T2[n, k])
                wabs = abs(Fraction(float(a1[n, g])) * int(T1[n, k])) + abs(Fraction(float(a2[n, g])) * int(T2[n, k]))
                acc += w * Fraction(float(x[m, k]))
                bnd += wabs * abs(Fraction(float(x[m, k])))
            assert abs(Fraction(y[m, n]) - acc) <= Fraction(1, 10 ** 13) * bnd
            assert abs(Fraction(B[m, n]) - bnd) <= Fraction(1, 10 ** 13) * bnd
    # one entry by hand: m=0, n=0: group0: a1=.5*(1.5-.25+3)=2.125, a2=.125*(-2+.25-3)=-.59375
    # group1: a1=.03125*(1+1.25)=.0703125, a2=-.25*(-.5-1)=.375  -> 1.9765625
    assert y[0, 0] == 1.9765625


# ---------------------------------------------------------------- unit-vector probes
def test_unit_vectors_return_columns():
    lin, _ = _small(20, 384, 1, key=3)
    W = oracle.reconstruct_dense(lin["T1"], lin["T2"], lin["a1"], lin["a2"])
    for j in (0, 1, 127, 128, 129, 255, 256, 383):
        e = np.zeros((1, 384), dtype=np.float16)
        e[0, j] = 1.0
        y, B = _fwd(lin, e)
        assert np.array_equal(y[0], W[:, j])
        assert np.array_equal(B[0], np.abs(lin["a1"][:, j // 128].astype(np.float64) * lin["T1"][:, j])
                              + np.abs(lin["a2"][:, j // 128].astype(np.float64) * lin["T2"][:, j]))


def test_unit_vector_hand_values():
    # column picked apart by hand: alpha1=0.5, alpha2=0.25, trits (+1,-1) -> 0.25 ; (0,+1) -> 0.25 ; (-1,-1) -> -0.75
    T1 = np.zeros((3, 128), dtype=np.int8)
    T2 = np.zeros((3, 128), dtype=np.int8)
    T1[:, 77] = [1, 0, -1]
    T2[:, 77] = [-1, 1, -1]
    a1 = np.full((3, 1), 0.5, dtype=np.float16)
    a2 = np.full((3, 1), 0.25, dtype=np.float16)
    e = np.zeros((1, 128), dtype=np.float16)
    e[0, 77] = 1.0
    y, _ = oracle.forward(T1, T2, a1, a2, e)
    assert y[0].tolist() == [0.25, 0.25, -0.75]


# ---------------------------------------------------------------- linearity, symmetry, locality
def test_linearity_in_x():
    lin, _ = _small(24, 512, 1, key=11)
    r = np.random.default_rng(5)
    x1 = r.standard_normal((2, 512))
    x2 = r.standard_normal((2, 512))
    a, b = 0.75, -2.5
    y1, B1 = _fwd(lin, x1)
    y2, B2 = _fwd(lin, x2)
    y12, _ = _fwd(lin, a * x1 + b * x2)
    assert np.all(np.abs(y12 - (a * y1 + b * y2)) <= 1e-13 * (abs(a) * B1 + abs(b) * B2))


def test_plane_swap_and_single_plane():
    lin, x = _small(24, 512, 2, key=13)
    y, B = _fwd(lin, x)
    ys, Bs = oracle.forward(lin["T2"], lin["T1"], lin["a2"], lin["a1"], x)
    assert np.all(np.abs(y - ys) <= 1e-13 * B)
    assert np.all(np.abs(B - Bs) <= 1e-13 * B)
    # second plane empty -> a plain single-plane ternary layer: einsum over groups
    Z = np.zeros_like(lin["T2"])
    y1, _ = oracle.forward(lin["T1"], Z, lin["a1"], lin["a2"], x)
    s = np.einsum("ngk,mgk->mng", lin["T1"].reshape(24, 4, 128).astype(np.float64),
                  x.astype(np.float64).reshape(2, 4, 128))
    ref = np.einsum("mng,ng->mn", s, lin["a1"].astype(np.float64))
    assert np.all(np.abs(y1 - ref) <= 1e-13 * B)
    # additivity over planes
    y2, _ = oracle.forward(Z, lin["T2"], lin["a1"], lin["a2"], x)
    assert np.all(np.abs(y - (y1 + y2)) <= 1e-13 * B)


def test_group_locality():
    lin, x = _small(16, 512, 1, key=17)
    xs = np.zeros_like(x)
    xs[:, 128:256] = x[:, 128:256]          # supported on group 1 only
    y, _ = _fwd(lin, xs)
    a1 = lin["a1"].copy()
    a2 = lin["a2"].copy()
    a1[:, [0, 2, 3]] = np.float16(123.0)
    a2[:, [0, 2, 3]] = np.float16(-55.0)
    yp, _ = oracle.forward(lin["T1"], lin["T2"], a1, a2, xs)
    assert np.array_equal(y, yp)
    # ... and does depend on its own group's scale
    a1[:, 1] = lin["a1"][:, 1] * np.float16(2)
    a2[:, 1] = lin["a2"][:, 1] * np.float16(2)
    y2, _ = oracle.forward(lin["T1"], lin["T2"], a1, a2, xs)
    assert np.allclose(y2, 2 * y, rtol=1e-14, atol=0)


def test_transpose_and_index_mistakes_would_show():
    # non-square, distinct rows/groups: y for row n must use row n's trits and scales only
    lin, x = _small(7, 256, 1, key=19)
    y, _ = _fwd(lin, x)
    for n in range(7):
        sub = {k: (v[n:n + 1] if isinstance(v, np.ndarray) else v) for k, v in lin.items()}
        yn, _ = oracle.forward(sub["T1"], sub["T2"], sub["a1"], sub["a2"], x)
        assert yn[0, 0] == y[0, n]
    # batch rows are independent
    x3 = workloads.make_x(3, 256, 90, 19)
    y3, _ = _fwd(lin, x3)
    for m in range(3):
        ym, _ = _fwd(lin, x3[m:m + 1])
        assert np.array_equal(ym[0], y3[m])


def test_integer_exact_case_is_order_free():
    lin, x = workloads.integer_exact_case(32, 1024, 2, 5)
    y, _ = _fwd(lin, x)
    yd = oracle.forward_dense(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x)
    assert np.array_equal(y, yd)
    assert np.array_equal(y.astype(np.float32).astype(np.float64), y)   # representable in fp32
    # integer arithmetic evaluation of the same thing
    s1 = x.astype(np.int64) @ lin["T1"].astype(np.int64).T
    s2 = x.astype(np.int64) @ lin["T2"].astype(np.int64).T
    assert np.array_equal(y, s1 / 32.0 + s2 / 128.0)


def test_threads_do_not_change_result():
    lin, x = _small(64, 512, 2, key=23)
    y1, B1 = _fwd(lin, x, threads=1)
    y4, B4 = _fwd(lin, x, threads=4)
    assert np.array_equal(y1, y4) and np.array_equal(B1, B4)


# ---------------------------------------------------------------- error paths
def test_rejects_bad_inputs():
    lin, x = _small(4, 256, 1, key=29)
    bad = lin["T1"].copy()
    bad[2, 100] = 2
    with pytest.raises(oracle.OracleError):
        oracle.forward(bad, lin["T2"], lin["a1"], lin["a2"], x)
    with pytest.raises(oracle.OracleError):
        oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x, group=96)
    with pytest.raises(oracle.OracleError):
        oracle.forward(lin["T1"], lin["T2"], lin["a1"], lin["a2"], x[:, :128])


# ---------------------------------------------------------------- canonical 2-bit storage
def test_pack_canonical_exhaustive():
    # all 81 four-trit patterns, byte value spelled out from the code table 00->0, 01->+1, 11->-1
    code = {0: 0b00, 1: 0b01, -1: 0b11}
    pats = [(a, b, c, d) for a in (-1, 0, 1) for b in (-1, 0, 1) for c in (-1, 0, 1) for d in (-1, 0, 1)]
    T = np.array(pats, dtype=np.int8)                     # [81, 4]
    P = oracle.pack_canonical(T)
    assert P.shape == (81, 1)
    for p, byte in zip(pats, P[:, 0]):
        want = code[p[0]] | code[p[1]] << 2 | code[p[2]] << 4 | code[p[3]] << 6
        assert int(byte) == want
    assert np.array_equal(oracle.unpack_canonical(P, 4), T)
    assert int(oracle.pack_canonical(np.array([[1, 0, -1, 1]], dtype=np.int8))[0, 0]) == 0x71


def test_pack_canonical_roundtrip_and_errors():
    T = workloads.make_trits(37, 640, 91)
    P = oracle.pack_canonical(T)
    assert P.shape == (37, 160) and P.dtype == np.uint8
    assert np.array_equal(oracle.unpack_canonical(P, 640), T)
    # every byte with a 10 field is rejected, every other byte accepted
    for b in range(256):
        has10 = any(((b >> (2 * j)) & 3) == 2 for j in range(4))
        arr = np.array([[b]], dtype=np.uint8)
        if has10:
            with pytest.raises(oracle.OracleError):
                oracle.unpack_canonical(arr, 4)
        else:
            oracle.unpack_canonical(arr, 4)
    bad = T.copy()
    bad[0, 0] = -2
    with pytest.raises(oracle.OracleError):
        oracle.pack_canonical(bad)


# ---------------------------------------------------------------- closed forms of the paper
def test_memory_model_golden():
    rows = [l.split() for l in open(os.path.join(GOLD, "memory_model.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 9
    for n, d, G, nbytes in rows:
        n, d, G, nbytes = int(n), int(d), int(G), int(nbytes)
        bits = oracle.model_bits(n, d, G)
        assert bits == 8 * nbytes
        assert Fraction(bits, n * d) == Fraction(17, 4)          # 4.25 bits per weight at G = 128
        T = workloads.make_trits(4, d, 92)
        assert oracle.pack_canonical(T).nbytes * 2 * n // 4 + 2 * n * (d // G) * 2 == nbytes


def test_storage_table_sanity():
    vals = dict(l.split() for l in open(os.path.join(GOLD, "storage_table3.txt")) if l.strip() and not l.startswith("#"))
    linear_w = 32 * sum(n * k for n, k in workloads.SHAPES_8B.values())
    other = 2 * 128256 * 4096 + 65 * 4096           # embeddings, lm_head, norms (LLaMA-3-8B)
    gib = 2.0 ** 30
    assert abs((linear_w + other) * 2 / gib - float(vals["fp16_gib"])) < 0.01
    ptqtp = (32 * sum(oracle.model_bits(n, k) for n, k in workloads.SHAPES_8B.values()) / 8 + other * 2) / gib
    assert abs(ptqtp - float(vals["ptqtp_gib"])) / float(vals["ptqtp_gib"]) < 0.05
