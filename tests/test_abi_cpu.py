"""CPU-only checks of the C ABI: the library loads, exports everything the header
declares, and its host-side argument validation answers without launching."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ptqtp.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ptqtp_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2509_16989_amd import binding
    if not os.path.exists(binding.lib_path()):
        import __graft_entry__
        __graft_entry__.build()
    return binding.raw()


def test_header_symbols_exported(lib):
    names = _declared()
    assert {"ptqtp_pack", "ptqtp_unpack", "ptqtp_gemv", "ptqtp_gemm_small", "ptqtp_packed_bytes",
            "ptqtp_workspace_bytes", "ptqtp_status_string", "ptqtp_version", "ptqtp_tune", "ptqtp_gemm",
            "ptqtp_gemv_batch", "ptqtp_gemv_batch_plan", "ptqtp_batch_items", "ptqtp_batch_plan_bytes",
            "ptqtp_quantize", "ptqtp_quantize_workspace_bytes", "ptqtp_gemm_batch", "ptqtp_gemm_batch_fused", "ptqtp_chain_plan_bytes",
            "ptqtp_chain_plan", "ptqtp_chain_run", "ptqtp_chain_run_batch", "ptqtp_gemm_route", "ptqtp_check_blob",
            "ptqtp_quantize_static"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in ptqtp.h but not exported"


def test_packed_bytes_closed_form(lib):
    # appendix memory model: N*K/2 bytes of planes + 4*N*K/G bytes of scales (+256-byte header)
    for n, k in [(1024, 1024), (4096, 4096), (1024, 4096), (14336, 4096), (4096, 14336),
                 (8192, 8192), (28672, 8192), (8192, 28672)]:
        assert lib.ptqtp_packed_bytes(1, n, k, 128) == 256 + n * k // 2 + 4 * n * k // 128
    # padding: N to 16 rows, K to 256 columns
    assert lib.ptqtp_packed_bytes(1, 1000, 1024, 128) == lib.ptqtp_packed_bytes(1, 1008, 1024, 128)
    assert lib.ptqtp_packed_bytes(1, 16, 128, 128) == 256 + 2176
    assert lib.ptqtp_packed_bytes(1, 16, 384, 128) == 256 + 2 * 2176
    # invalid
    assert lib.ptqtp_packed_bytes(1, 16, 100, 128) == 0
    assert lib.ptqtp_packed_bytes(1, 16, 256, 64) == 0
    assert lib.ptqtp_packed_bytes(0, 16, 256, 128) == 0
    assert lib.ptqtp_packed_bytes(1, -4, 256, 128) == 0
    assert lib.ptqtp_workspace_bytes(1, 4096, 4096, 128) == 0


def test_batch_plan_validation(lib):
    from paper_2509_16989_amd.binding import _Linear
    arr = (_Linear * 3)()
    arr[0] = _Linear(0x10000, 0x20000, 0x30000, 4096, 4096)
    arr[1] = _Linear(0x10000, 0x20000, 0x30000, 1000, 1024)
    arr[2] = _Linear(0x10000, 0x20000, 0x30000, 16, 128)
    items = 256 + 64 + 16           # ceil(N/16) per entry, rounded up to a multiple of sixteen
    assert lib.ptqtp_batch_items(arr, 3, 128) == items
    assert lib.ptqtp_batch_plan_bytes(arr, 3, 128) == 64 + 3 * 48 + 4 * items
    assert lib.ptqtp_batch_items(arr, 0, 128) == 0
    assert lib.ptqtp_batch_items(arr, 3, 64) == 0
    assert lib.ptqtp_batch_items(None, 3, 128) == 0
    fake = ctypes.c_void_p(0x40000)
    assert lib.ptqtp_gemv_batch_plan(arr, 3, 0, 128, fake, 10, None) == 4          # plan buffer too small
    assert lib.ptqtp_gemv_batch_plan(arr, 3, 9, 128, fake, 1 << 20, None) == 5
    assert lib.ptqtp_gemv_batch_plan(arr, 3, 0, 128, None, 1 << 20, None) == 1
    arr[1].K = 1000
    assert lib.ptqtp_gemv_batch_plan(arr, 3, 0, 128, fake, 1 << 20, None) == 2
    arr[1].K = 1024
    arr[2].x = 0
    assert lib.ptqtp_gemv_batch_plan(arr, 3, 0, 128, fake, 1 << 20, None) == 1
    arr[2].x = 0x20002
    assert lib.ptqtp_gemv_batch_plan(arr, 3, 0, 128, fake, 1 << 20, None) == 6
    assert lib.ptqtp_gemv_batch(None, 5, None) == 1
    assert lib.ptqtp_gemv_batch(fake, 0, None) == 2


def test_chain_plan_validation(lib):
    from paper_2509_16989_amd.binding import _Stage
    def stages():
        arr = (_Stage * 3)()
        arr[0] = _Stage(0x10000, 0x20000, 0x30000, None, 4096, 4096, 0, 1, 0, 0)
        arr[1] = _Stage(0x10000, 0x30000, 0x40000, 0x20000, 960, 4096, 1, 1, 1, 0)      # gated pair: 960/32 = 30 items
        arr[2] = _Stage(0x10000, 0x40000, 0x50000, None, 100, 512 - 128, 0, 0, 5, 0)     # levels need not be dense
        return arr
    arr = stages()
    items = 256 + 30 + 7
    want = 256 + 3 * 72 + 4 * items      # header, table, item map
    assert lib.ptqtp_chain_plan_bytes(arr, 3, 128) == (want + 255) // 256 * 256
    assert lib.ptqtp_chain_plan_bytes(arr, 0, 128) == 0
    assert lib.ptqtp_chain_plan_bytes(arr, 3, 64) == 0
    assert lib.ptqtp_chain_plan_bytes(None, 3, 128) == 0
    fake = ctypes.c_void_p(0x100000)
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 16, None) == 4
    assert lib.ptqtp_chain_plan(arr, 3, 128, None, 1 << 20, None) == 1
    assert lib.ptqtp_chain_plan(arr, 3, 128, ctypes.c_void_p(0x100010), 1 << 20, None) == 6
    arr = stages(); arr[1].N = 944          # gated stage: N must be a multiple of 32
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 1 << 20, None) == 2
    arr = stages(); arr[2].level = 0        # levels must not decrease
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 1 << 20, None) == 2
    arr = stages(); arr[0].epilogue = 7
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 1 << 20, None) == 2
    arr = stages(); arr[0].y_dtype = 3
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 1 << 20, None) == 5
    arr = stages(); arr[1].K = 4000
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 1 << 20, None) == 2
    arr = stages(); arr[2].y = 0
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 1 << 20, None) == 1
    arr = stages(); arr[1].residual = 0x20002
    assert lib.ptqtp_chain_plan(arr, 3, 128, fake, 1 << 20, None) == 6
    arr = stages()
    assert lib.ptqtp_chain_run(arr, 3, 128, None, None) == 1
    assert lib.ptqtp_chain_run(arr, 3, 128, ctypes.c_void_p(0x100010), None) == 6
    assert lib.ptqtp_chain_run_batch(arr, 3, 128, 0, None) == 2
    assert lib.ptqtp_chain_run_batch(arr, 3, 128, 65537, None) == 2
    assert lib.ptqtp_chain_run_batch(None, 3, 128, 4, None) == 1
    arr[1].N = 944
    assert lib.ptqtp_chain_run(arr, 3, 128, fake, None) == 2
    assert lib.ptqtp_chain_run_batch(arr, 3, 128, 4, None) == 2


def test_quantize_validation(lib):
    fake = ctypes.c_void_p(0x10000)
    assert lib.ptqtp_quantize_workspace_bytes(4096, 4096, 128) == 256 + 4096 * 32 * 32
    assert lib.ptqtp_quantize_workspace_bytes(4096, 4000, 128) == 0
    assert lib.ptqtp_quantize_workspace_bytes(4096, 4096, 64) == 0
    big = 1 << 30
    args = lambda **k: [k.get("W", fake), k.get("N", 64), k.get("K", 256), k.get("group", 128), k.get("iters", 50),
                        ctypes.c_double(k.get("eps", 1e-4)), fake, fake, fake, fake, None, k.get("ws", fake),
                        k.get("wsb", big), None]
    assert lib.ptqtp_quantize(*args(W=None)) == 1
    assert lib.ptqtp_quantize(*args(ws=None)) == 1
    assert lib.ptqtp_quantize(*args(group=64)) == 3
    assert lib.ptqtp_quantize(*args(K=200)) == 2
    assert lib.ptqtp_quantize(*args(N=1 << 20, K=1 << 18)) == 2          # N * K above 2^37
    assert lib.ptqtp_quantize_workspace_bytes(1 << 20, 1 << 18, 128) == 0
    assert lib.ptqtp_quantize_workspace_bytes(1 << 20, 1 << 17, 128) == 256 + (1 << 30) * 32
    assert lib.ptqtp_quantize(*args(iters=-1)) == 2
    assert lib.ptqtp_quantize(*args(eps=-1.0)) == 2
    assert lib.ptqtp_quantize(*args(eps=float("nan"))) == 2
    assert lib.ptqtp_quantize(*args(wsb=100)) == 4
    assert lib.ptqtp_quantize(*args(ws=ctypes.c_void_p(0x10010))) == 6


def test_check_blob_and_static_quantizer_validation(lib):
    fake, status = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000)
    need = lib.ptqtp_packed_bytes(1, 64, 256, 128)
    assert lib.ptqtp_check_blob(None, need, 64, 256, 128, status, None) == 1
    assert lib.ptqtp_check_blob(fake, need, 64, 256, 128, None, None) == 1
    assert lib.ptqtp_check_blob(fake, need, 64, 200, 128, status, None) == 2
    assert lib.ptqtp_check_blob(fake, need, 64, 256, 64, status, None) == 3
    assert lib.ptqtp_check_blob(fake, need - 1, 64, 256, 128, status, None) == 4
    assert lib.ptqtp_check_blob(ctypes.c_void_p(0x10080), need, 64, 256, 128, status, None) == 6
    assert lib.ptqtp_check_blob(fake, need, 64, 256, 128, ctypes.c_void_p(0x20002), None) == 6
    # the static-workspace quantizer refuses on the host what its array cannot hold, and bad arguments as ptqtp_quantize does
    args = lambda **k: [k.get("W", fake), k.get("N", 64), k.get("K", 256), k.get("group", 128), k.get("iters", 50),
                        ctypes.c_double(k.get("eps", 1e-4)), fake, fake, fake, fake, None, None]
    assert lib.ptqtp_quantize_static(*args(W=None)) == 1
    assert lib.ptqtp_quantize_static(*args(group=64)) == 3
    assert lib.ptqtp_quantize_static(*args(K=200)) == 2
    assert lib.ptqtp_quantize_static(*args(iters=-1)) == 2
    assert lib.ptqtp_quantize_static(*args(N=16385, K=4096)) == 4
    assert lib.ptqtp_quantize_static(*args(N=1 << 20, K=1 << 17)) == 4


def test_size_limits(lib):
    """N and K up to 2^30 each, and at most 2^27 records per layer: beyond that no grid or count fits 32 bits."""
    assert lib.ptqtp_packed_bytes(1, 1 << 21, 1 << 17, 128) == 256 + (1 << 26) * 2176     # 2^17 x 2^9 records
    assert lib.ptqtp_packed_bytes(1, 1 << 22, 1 << 17, 128) == 256 + (1 << 27) * 2176     # the limit itself
    assert lib.ptqtp_packed_bytes(1, (1 << 22) + 1, 1 << 17, 128) == 0
    assert lib.ptqtp_packed_bytes(1, 1 << 30, 1 << 30, 128) == 0
    assert lib.ptqtp_packed_bytes(1, (1 << 30) + 16, 128, 128) == 0
    route = (ctypes.c_int32 * 4)()
    assert lib.ptqtp_gemm_route(512, 1 << 30, 1 << 30, 128, 0, route) == 2


def test_binding_rejects_short_buffers_before_any_launch():
    """The kernels trust N and K, so the binding compares them with the buffers it is handed (host tensors suffice
    to show it: the size checks come before the device checks)."""
    import torch
    import paper_2509_16989_amd as ptq
    N, K = 64, 256
    need = ptq.ptqtp_packed_bytes(1, N, K)
    short = torch.zeros(need - 1, dtype=torch.uint8)
    x = torch.zeros(K, dtype=torch.float16)
    with pytest.raises(ptq.PtqtpError) as e:
        ptq.ptqtp_gemv(short, x, N, K)
    assert e.value.status == 4
    with pytest.raises(ptq.PtqtpError) as e:
        ptq.ptqtp_gemm(short, x.reshape(1, K), N, K)
    assert e.value.status == 4
    with pytest.raises(ptq.PtqtpError) as e:
        ptq.ptqtp_unpack(short, N, K)
    assert e.value.status == 4
    full = torch.zeros(need, dtype=torch.uint8)
    with pytest.raises(ptq.PtqtpError) as e:                   # output of the wrong size
        ptq.ptqtp_gemm(full, x.reshape(1, K), N, K, out=torch.zeros(N - 1))
    assert e.value.status == 2
    with pytest.raises(ptq.PtqtpError) as e:
        ptq.ptqtp_gemv_batch_plan([(short, x, torch.zeros(N), N, K)])
    assert e.value.status == 4
    with pytest.raises(ptq.PtqtpError) as e:                   # y holds fewer tokens than x
        ptq.ptqtp_gemv_batch_plan([(full, torch.zeros(2 * K, dtype=torch.float16), torch.zeros(N), N, K)])
    assert e.value.status == 2
    with pytest.raises(ptq.PtqtpError) as e:
        ptq.ptqtp_chain_plan([dict(packed=short, x=x, y=torch.zeros(N), N=N, K=K)])
    assert e.value.status == 4
    with pytest.raises(ptq.PtqtpError) as e:                   # a gated stage writes N/2 outputs: room for none here
        ptq.ptqtp_chain_plan([dict(packed=full, x=x, y=torch.zeros(N // 2 - 1), N=N, K=K, epilogue=ptq.PTQTP_EPI_SWIGLU)])
    assert e.value.status == 2


def test_status_strings_and_version(lib):
    assert lib.ptqtp_version() >= 100
    seen = set()
    for s in range(8):
        msg = lib.ptqtp_status_string(s)
        assert msg and msg not in seen
        seen.add(msg)
    assert lib.ptqtp_status_string(99) == b"unknown status"


def test_argument_validation_without_launch(lib):
    fake = ctypes.c_void_p(0x10000)          # aligned, never dereferenced on these paths
    N, K = 64, 256
    # null pointers
    assert lib.ptqtp_gemv(None, fake, fake, 0, 1, N, K, 128, None, 0, None) == 1
    assert lib.ptqtp_pack(None, fake, fake, fake, 1, N, K, 128, fake, 10 ** 9, None, None) == 1
    assert lib.ptqtp_unpack(None, 1, N, K, 128, fake, fake, fake, fake, None) == 1
    # shapes
    assert lib.ptqtp_gemv(fake, fake, fake, 0, 2, N, K, 128, None, 0, None) == 2      # gemv needs M == 1
    assert lib.ptqtp_gemv(fake, fake, fake, 0, 1, N, 200, 128, None, 0, None) == 2    # K % group
    assert lib.ptqtp_gemm_small(fake, fake, fake, 0, 65, N, K, 128, None, 0, None) == 2
    assert lib.ptqtp_gemm_small(fake, fake, fake, 0, 0, N, K, 128, None, 0, None) == 2
    # empty layers and the largest batch
    assert lib.ptqtp_gemv(fake, fake, fake, 0, 1, 0, K, 128, None, 0, None) == 2
    assert lib.ptqtp_gemv(fake, fake, fake, 0, 1, N, 0, 128, None, 0, None) == 2
    assert lib.ptqtp_gemm(fake, fake, fake, 0, 65537, N, K, 128, None, 0, None) == 2
    assert lib.ptqtp_packed_bytes(1, 0, K, 128) == 0 and lib.ptqtp_packed_bytes(1, N, 0, 128) == 0
    # the fused-planes flag belongs to ptqtp_gemm only
    assert lib.ptqtp_gemv(fake, fake, fake, 16, 1, N, K, 128, None, 0, None) == 5
    assert lib.ptqtp_gemm_small(fake, fake, fake, 16 | 1, 4, N, K, 128, None, 0, None) == 5
    assert lib.ptqtp_gemm(fake, fake, fake, 16 | 2, 300, N, K, 128, None, 0, None) == 5
    # group, dtype, size, alignment
    assert lib.ptqtp_gemv(fake, fake, fake, 0, 1, N, K, 64, None, 0, None) == 3
    assert lib.ptqtp_gemv(fake, fake, fake, 7, 1, N, K, 128, None, 0, None) == 5
    assert lib.ptqtp_pack(fake, fake, fake, fake, 1, N, K, 128, fake, 100, None, None) == 4
    assert lib.ptqtp_gemv(ctypes.c_void_p(0x10010), fake, fake, 0, 1, N, K, 128, None, 0, None) == 6
    assert lib.ptqtp_gemv(fake, ctypes.c_void_p(0x10002), fake, 0, 1, N, K, 128, None, 0, None) == 6
    # tuning hook
    assert lib.ptqtp_tune(b"small_waves", 8) == 0
    assert lib.ptqtp_tune(b"small_waves", 0) == 0
    assert lib.ptqtp_tune(b"small_rows", 3) == 2
    assert lib.ptqtp_tune(b"stream_depth", 3) == 2
    assert lib.ptqtp_tune(b"stream_waves", 17) == 2
    assert lib.ptqtp_tune(b"stream_waves", 0) == 0
    assert lib.ptqtp_tune(b"nonsense", 1) == 2


# ---------------------------------------------------------------- which kernels a shape gets (host logic)
def _route(lib, M, N, K, y_dtype=0):
    r = (ctypes.c_int32 * 4)()
    assert lib.ptqtp_gemm_route(M, N, K, 128, y_dtype, r) == 0
    return tuple(r)


def test_gemm_route_regimes(lib):
    STREAM, SMALL, CHUNKS, TILE = 0, 1, 2, 3
    assert _route(lib, 1, 4096, 4096)[0] == STREAM
    # few tokens, or few rows: the small-batch kernel (in chunks of 64 tokens above 64)
    for M in (2, 16, 32):
        assert _route(lib, M, 14336, 4096)[0] == SMALL
    assert _route(lib, 64, 4096, 4096)[0] == SMALL
    assert _route(lib, 96, 4096, 4096)[0] == CHUNKS
    assert _route(lib, 64, 328, 2304)[0] == SMALL
    # a wide layer fills the chip with 64 x 64 tiles from a few dozen tokens on
    assert _route(lib, 64, 14336, 4096) == (TILE, 4, 0, -1)
    assert _route(lib, 128, 14336, 4096)[:2] == (TILE, 3)
    # short prompts on 8B shapes: the smaller tiles; long ones: the big tiles
    assert _route(lib, 256, 4096, 4096) == (TILE, 4, 0, -1)
    assert _route(lib, 512, 4096, 4096) == (TILE, 3, 0, -1)
    assert _route(lib, 512, 1024, 4096) == (TILE, 4, 0, -1)
    assert _route(lib, 2048, 1024, 8192)[1] in (3, 4)
    assert _route(lib, 2048, 8192, 28672)[1] in (0, 1, 2)
    # 70B gate at 2048 tokens: 896 tiles of 256 x 256 = 3.5 rounds of 256 CUs -> three whole rounds, then smaller tiles
    path, kind, split, second = _route(lib, 2048, 28672, 8192)
    assert (path, kind) == (TILE, 0) and split == 96 * 16 and second in (1, 2, 3)
    # every tile launch covers whole row blocks of its own tile: the split is a multiple of 16 row tiles
    for M in (256, 300, 777, 2048, 5000):
        for N in (1000, 4096, 9216, 28672):
            r = _route(lib, M, N, 4096)
            assert r[0] == TILE and 0 <= r[1] <= 4 and r[2] % 16 == 0 and r[2] < (N + 15) // 16
            assert (r[2] == 0) == (r[3] == -1)
    # the fused-plane flag only counts from 256 tokens on, and never changes the regime
    assert _route(lib, 64, 4096, 4096, 16) == _route(lib, 64, 4096, 4096)
    assert _route(lib, 512, 4096, 4096, 16)[0] == TILE


def test_gemm_route_follows_tuning_and_rejects_bad_shapes(lib):
    r = (ctypes.c_int32 * 4)()
    try:
        assert lib.ptqtp_tune(b"tile", 1) == 0
        assert _route(lib, 2, 328, 2304)[0] == 3
        assert lib.ptqtp_tune(b"tile", -1) == 0
        assert _route(lib, 64, 14336, 4096)[0] == 1 and _route(lib, 200, 14336, 4096)[0] == 2
        assert lib.ptqtp_tune(b"tile", 0) == 0
        for variant, kind in ((1, 1), (2, 2), (3, 0), (4, 3), (5, 4)):
            assert lib.ptqtp_tune(b"tile_variant", variant) == 0
            assert _route(lib, 512, 4096, 4096) == (3, kind, 0, -1)
        assert lib.ptqtp_tune(b"tile_variant", 6) == 2
    finally:
        lib.ptqtp_tune(b"tile", 0)
        lib.ptqtp_tune(b"tile_variant", 0)
    assert lib.ptqtp_gemm_route(4, 4096, 4096, 128, 0, None) == 1
    assert lib.ptqtp_gemm_route(4, 4096, 4000, 128, 0, r) == 2
    assert lib.ptqtp_gemm_route(4, 4096, 4096, 64, 0, r) == 3
    assert lib.ptqtp_gemm_route(0, 4096, 4096, 128, 0, r) == 2
