"""GPU parity of the GEMM when the tiles of the last, partial round are shared
along K through the caller's workspace (two pieces per tile, partial sums in
FP32, the second arrival adds them up): same oracle, same bars as the plain
path.  With small-integer codes and power-of-two scales every partial sum is
exact, so the shared result must equal the oracle -- and the result computed
without a workspace -- bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from tests._gpu_util import announce, dev, host, normwise

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL_F32 = 1e-4

TABLE = np.array([0x00, 0x38, 0x40, 0xB8, 0xC0, 0x80], dtype=np.uint8)  # 0, 1, 2, -1, -2, -0


def _rand_codes(rng, shape):
    c = rng.integers(0, 0x7F, size=shape).astype(np.uint8)
    return c | (rng.integers(0, 2, size=shape) << 7).astype(np.uint8)


def _ws(ds3, variant, m, n, k, mode=0):
    nbytes = ds3.ds3_gemm_workspace_bytes_v(variant, m, n, k, mode)
    assert nbytes > 0, "this shape was chosen to share its tail tiles"
    # arbitrary contents but for the counters, which the init call prepares
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda:0")
    assert ds3._L().ds3_gemm_workspace_init(ws.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream) == 0
    return ws


# shapes whose tile count leaves a partial round for the given variant on a 256-CU chip
SHARED = [
    (0, (1024, 1024, 1024)),     # 16 tiles of 256x256, 2 per XCD, 8 K-steps: halves
    (0, (512, 512, 4096)),       # 4 tiles, one per XCD for half of the XCDs (the others get none)
    (0, (300, 576, 1152)),       # ragged in M and N, 9 K-steps: pieces of 5 and 4
    (0, (2048, 9216, 512)),      # a full round of whole tiles first, then 4 shared tiles per XCD
    (1, (1024, 640, 768)),       # 256x128 tiles, three LDS stages
    (1, (130, 257, 256)),        # two K-steps only: one each
    (2, (640, 384, 1280)),       # 128x128 tiles, two workgroups per CU
    (2, (17, 130, 384)),
]


@pytest.mark.parametrize("variant,shape", SHARED)
def test_shared_tiles_exact(ds3, variant, shape):
    m, n, k = shape
    announce(f"share-K exact variant {variant} {shape}")
    rng = np.random.default_rng(61)
    a, b = TABLE[rng.integers(0, 6, (m, k))], TABLE[rng.integers(0, 6, (n, k))]
    sa = np.ldexp(1.0, rng.integers(-2, 2, (m, k // 128))).astype(np.float32)
    sb = np.ldexp(1.0, rng.integers(-1, 3, ((n + 127) // 128, k // 128))).astype(np.float32)
    ref = orc.gemm_fp8_bs(a, sa, b, sb)
    ws = _ws(ds3, variant, m, n, k)
    args = (dev(a), dev(sa), dev(b), dev(sb))
    c = host(ds3.ds3_gemm_fp8_bs(*args, out_dtype=torch.float32, variant=variant, workspace=ws))
    bad = np.argwhere(c.astype(np.float64) != ref)
    assert bad.size == 0, f"{bad.shape[0]} mismatches, first {bad[0]}: {c[tuple(bad[0])]} vs {ref[tuple(bad[0])]}"
    plain = host(ds3.ds3_gemm_fp8_bs(*args, out_dtype=torch.float32, variant=variant, workspace=None))
    assert np.array_equal(c, plain)
    # the workspace is left ready: a second call on the same, uncleared workspace and a BF16 output
    c16 = host(ds3.ds3_gemm_fp8_bs(*args, variant=variant, workspace=ws))
    assert np.array_equal(c16.astype(np.float64), orc.round_to_bf16(ref))
    # per-row weight scales with accumulation into FP32 (the weight-gradient form)
    sbr = np.ldexp(1.0, rng.integers(-1, 3, (n, k // 128))).astype(np.float32)
    c0 = rng.integers(-4, 5, (m, n)).astype(np.float32)
    ref2 = orc.gemm_fp8_bs(a, sa, b, sbr, sb_per_row=True, c_in=c0)
    wsr = _ws(ds3, variant, m, n, k, ds3.DS3_BSCALE_PER_ROW)
    cacc = torch.zeros((m, (n + 7) // 8 * 8), dtype=torch.float32, device="cuda:0")[:, :n]   # leading dimension % 4
    cacc.copy_(dev(c0))
    ds3.ds3_gemm_fp8_bs(args[0], args[1], args[2], dev(sbr), sb_mode=ds3.DS3_BSCALE_PER_ROW, c=cacc, accumulate=True,
                        variant=variant, workspace=wsr)
    assert np.array_equal(host(cacc).astype(np.float64), ref2)


@pytest.mark.parametrize("variant,shape", [(0, (1024, 1280, 2048)), (1, (777, 640, 1024)), (2, (640, 384, 1280))])
def test_shared_tiles_random_codes(ds3, variant, shape):
    m, n, k = shape
    announce(f"share-K random variant {variant} {shape}")
    rng = np.random.default_rng(62)
    a, b = _rand_codes(rng, (m, k)), _rand_codes(rng, (n, k))
    sa = np.exp(rng.standard_normal((m, k // 128))).astype(np.float32)
    sb = np.exp(rng.standard_normal(((n + 127) // 128, k // 128))).astype(np.float32)
    ref = orc.gemm_fp8_bs(a, sa, b, sb)
    ws = _ws(ds3, variant, m, n, k)
    args = (dev(a), dev(sa), dev(b), dev(sb))
    c32 = host(ds3.ds3_gemm_fp8_bs(*args, out_dtype=torch.float32, variant=variant, workspace=ws))
    c16 = ds3.ds3_gemm_fp8_bs(*args, variant=variant, workspace=ws)
    e32, e16 = normwise(c32, ref), normwise(host(c16), ref)
    print(f"{shape} variant {variant}: fp32 {e32:.3e} bf16 {e16:.3e}")
    assert e32 <= TOL_F32 and e16 <= TOL_BF16
    # the order of the two arrivals varies from run to run; the bits must not
    for _ in range(3):
        assert torch.equal(c16, ds3.ds3_gemm_fp8_bs(*args, variant=variant, workspace=ws))
    # sharing changes the order of the FP32 additions only
    plain = host(ds3.ds3_gemm_fp8_bs(*args, out_dtype=torch.float32, variant=variant, workspace=None))
    assert normwise(c32, plain.astype(np.float64)) <= 1e-6


def test_one_workspace_serves_different_shapes_in_turn(ds3):
    """Counters are left at zero by every call, partial tiles are overwritten before they are read."""
    announce("share-K workspace reuse")
    rng = np.random.default_rng(63)
    shapes = [(1024, 1024, 1024), (300, 576, 1152), (1024, 1024, 1024), (512, 512, 4096)]
    ws = ds3.new_gemm_workspace(max(ds3.ds3_gemm_workspace_bytes_v(0, *s) for s in shapes), "cuda:0")
    for m, n, k in shapes:
        a, b = TABLE[rng.integers(0, 6, (m, k))], TABLE[rng.integers(0, 6, (n, k))]
        sa = np.ldexp(1.0, rng.integers(-2, 2, (m, k // 128))).astype(np.float32)
        sb = np.ldexp(1.0, rng.integers(-1, 3, ((n + 127) // 128, k // 128))).astype(np.float32)
        c = host(ds3.ds3_gemm_fp8_bs(dev(a), dev(sa), dev(b), dev(sb), out_dtype=torch.float32, variant=0, workspace=ws))
        assert np.array_equal(c.astype(np.float64), orc.gemm_fp8_bs(a, sa, b, sb)), (m, n, k)


def test_empty_inner_dimension(ds3):
    """K = 0: the sum is empty -- zero without accumulation, untouched with it; padding columns stay."""
    announce("K = 0")
    L = ds3._L()
    for dt, ct in ((torch.bfloat16, ds3.DS3_BF16), (torch.float32, ds3.DS3_F32)):
        c = torch.full((37, 72), 3.0, dtype=dt, device="cuda:0")
        st = L.ds3_gemm_fp8_bs(37, 70, 0, None, 0, None, 0, 0, None, 0, None, 0, 0, 0, c.data_ptr(), ct, 72, 0, None, 0,
                               torch.cuda.current_stream().cuda_stream)
        assert st == 0
        h = host(c)
        assert np.all(h[:, :70] == 0) and np.all(h[:, 70:] == 3.0)
    c = torch.full((8, 8), 3.0, dtype=torch.float32, device="cuda:0")
    assert L.ds3_gemm_fp8_bs(8, 8, 0, None, 0, None, 0, 0, None, 0, None, 0, 0, 0, c.data_ptr(), ds3.DS3_F32, 8, 1, None, 0,
                             torch.cuda.current_stream().cuda_stream) == 0
    assert np.all(host(c) == 3.0)
