"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pkg():
    import paper_2412_19437_amd as p
    if not os.path.exists(p.LIB_PATH):
        from paper_2412_19437_amd.build import build_library
        build_library(verbose=False)
    return p


def test_every_declared_symbol_is_exported(pkg):
    header = open(os.path.join(ROOT, "include", "ds3.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ds3_[a-z0-9_]+)\s*\(", header))
    assert {"ds3_quant_act_1x128", "ds3_quant_act_128x1", "ds3_quant_w_128x128",
            "ds3_gemm_fp8_bs", "ds3_grouped_gemm_fp8_bs"} <= declared
    lib = ctypes.CDLL(pkg.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(pkg.SYMBOLS)


def test_status_strings(pkg):
    seen = {pkg.status_string(i) for i in range(8)}
    assert len(seen) == 8 and pkg.status_string(0) == "ok" and pkg.status_string(99) == "unknown status"


def test_quantizers_reject_bad_arguments_on_the_host(pkg):
    L = pkg._L()
    buf = (ctypes.c_uint8 * 4096)()
    p = ctypes.addressof(buf)                      # host memory: never dereferenced, checks come first
    p = (p + 15) & ~15
    q = L.ds3_quant_act_1x128
    assert q(None, 1, 4, 128, 128, p, 128, p, 1, 4, None) == 1          # NULL
    assert q(p, 7, 4, 128, 128, p, 128, p, 1, 4, None) == 4             # dtype
    assert q(p, 1, -1, 128, 128, p, 128, p, 1, 4, None) == 2            # negative rows
    assert q(p, 1, 4, 128, 64, p, 128, p, 1, 4, None) == 2              # ld < cols
    assert q(p, 1, 4, 132, 136, p, 144, p, 1, 4, None) == 3             # cols not a multiple of 8 (BF16)
    assert q(p + 2, 1, 4, 128, 128, p, 128, p, 1, 4, None) == 3         # misaligned pointer
    assert q(p, 1, 0, 128, 128, None, 128, None, 1, 4, None) == 0       # empty: no-op even with NULLs
    w = L.ds3_quant_w_128x128
    assert w(p, 0, 4, 130, 132, p, 144, p, None) == 3                   # FP32: cols % 4
    assert w(p, 0, 4, 128, 128, None, 128, p, None) == 1
    t = L.ds3_quant_act_128x1
    assert t(p, 1, 130, 128, 128, p, 128, p, 1, 128, None) == 2         # ldq < rows
    assert t(p, 1, 130, 128, 128, p, 136, p, 1, 128, None) == 3         # ldq % 16


def test_gemm_rejects_bad_arguments_on_the_host(pkg):
    L = pkg._L()
    buf = (ctypes.c_uint8 * 4096)()
    p = (ctypes.addressof(buf) + 15) & ~15
    g = L.ds3_gemm_fp8_bs

    def call(M=16, N=16, K=128, a=p, lda=128, sa=p, b=p, ldb=128, sb=p, mode=0, c=p, ct=1, ldc=16, acc=0):
        return g(M, N, K, a, lda, sa, 1, M, b, ldb, sb, 1, 1, mode, c, ct, ldc, acc, None, 0, None)

    assert call(K=100) == 2                       # K % 128
    assert call(a=None) == 1
    assert call(lda=64) == 2
    assert call(lda=136) == 3
    assert call(ldc=18) == 3
    assert call(ct=1, acc=1) == 4                 # accumulate into BF16
    assert call(mode=5) == 4
    assert call(M=0, a=None, c=None) == 0         # empty
    assert call(M=-1) == 2
    gg = L.ds3_grouped_gemm_fp8_bs
    assert gg(2, None, 16, 16, 128, p, 128, p, 1, 16, p, 128, p, p, 1, 16, None, 0, None) == 1
    assert gg(0, None, 16, 16, 128, p, 128, p, 1, 16, p, 128, p, p, 1, 16, None, 0, None) == 0
    assert gg(1024, p, 16, 16, 128, p, 128, p, 1, 16, p, 128, p, p, 1, 16, None, 0, None) == 5   # more than 1023 experts
    assert L.ds3_gemm_fp8_bs_v(99, 16, 16, 128, p, 128, p, 1, 16, p, 128, p, 1, 1, 0, p, 1, 16, 0, None, 0, None) == 5
    assert L.ds3_swiglu(p, 4, 12, 24, p, 16, None) == 3
    assert L.ds3_swiglu(None, 4, 16, 32, p, 16, None) == 1


def test_gemm_workspace_contract_on_the_host(pkg):
    """The size query answers without a GPU (it assumes 256 compute units then), a workspace
    that is too small or misaligned is refused before any launch, and none at all is accepted."""
    L = pkg._L()
    buf = (ctypes.c_uint8 * 4096)()
    p = (ctypes.addressof(buf) + 15) & ~15
    counters = (8 * 64 + 64) * 4                   # arrival counters of shared tiles + the grouped walk's tile queue
    assert L.ds3_grouped_gemm_workspace_bytes() == counters

    def need(shared_tiles_per_xcd, tile_floats):   # arrival counters + two FP32 partial tiles per shared tile
        return counters + 8 * shared_tiles_per_xcd * 2 * tile_floats * 4

    # 8192 x 576 on 256 x 256 tiles: 32 x 3 = 96 tiles for 256 workgroups, 12 per XCD: shared (two pieces each)
    assert pkg.ds3_gemm_workspace_bytes_v(0, 8192, 576, 7168) == need(12, 256 * 256)
    # 4096 x 18432: 1152 tiles, half a round is left over: the half-tile split serves it, no workspace
    assert pkg.ds3_gemm_workspace_bytes(4096, 18432, 7168) == 0
    # 8192 x 24576: 32 x 96 = 3072 tiles, 12 full rounds: nothing to share
    assert pkg.ds3_gemm_workspace_bytes_v(0, 8192, 24576, 1536) == 0
    # 2048 x 9216: 288 tiles: a full round and 4 tiles per XCD, an eighth of a round: shared
    assert pkg.ds3_gemm_workspace_bytes_v(0, 2048, 9216, 512) == need(4, 256 * 256)
    # 256 x 128 tiles (the weight-gradient form's large-shape default): 640 x 1024 -> 5 x 4 = 20 tiles, at most 3 per XCD
    assert pkg.ds3_gemm_workspace_bytes_v(1, 640, 1024, 768, pkg.DS3_BSCALE_PER_ROW) == need(3, 256 * 128)
    # few tiles: the default choice is 128 x 128 tiles, 5 x 8 = 40 of them, 5 per XCD
    assert pkg.ds3_gemm_workspace_bytes_v(-1, 640, 1024, 768, pkg.DS3_BSCALE_PER_ROW) == need(5, 128 * 128)
    assert pkg.ds3_gemm_workspace_bytes(0, 16, 128) == 0 and pkg.ds3_gemm_workspace_bytes(16, 16, 100) == 0
    assert pkg.ds3_gemm_workspace_bytes_v(9, 8192, 576, 7168) == 0
    # the statically allocated workspace of the entry point that allocates nothing covers the largest need
    assert pkg._L().ds3_gemm_noalloc_scratch_bytes() == need(19, 256 * 256)
    need = need(12, 256 * 256)

    def call(ws, nbytes, M=8192, N=576, K=7168):
        return L.ds3_gemm_fp8_bs_v(0, M, N, K, p, K, p, 1, M, p, K, p, K // 128, 1, 0, p, 1, N, 0, ws, nbytes, None)

    assert call(p, need - 1) == 7                 # DS3_ERR_WORKSPACE
    assert call(p, 0) == 7
    assert call(p + 4, need) == 3                 # misaligned workspace
    assert pkg.status_string(7).startswith("workspace")
    # the grouped calls: a workspace smaller than their tile queue's counters is refused, a misaligned one too
    def grouped(ws, nbytes):
        return L.ds3_grouped_gemm_fp8_bs(2, p, 512, 256, 256, p, 256, p, 1, 512, p, 256, p, p, 1, 256, ws, nbytes, None)

    def grouped_swiglu(ws, nbytes):
        return L.ds3_grouped_gemm_swiglu_quant_fp8_bs(2, p, 512, 128, 256, p, 256, p, 1, 512, p, 256, p, p, 128, p, 1, 512,
                                                      ws, nbytes, None)
    for f in (grouped, grouped_swiglu):
        assert f(p, counters - 1) == 7 and f(p, 0) == 7
        assert f(p + 4, counters) == 3


def test_tail_share_steps_never_cuts_a_tile_in_three(pkg):
    """Brute force over the small cases: the chosen run length q covers the tail with at most
    `workgroups` runs, is minimal with that property, and no tile meets more than two runs."""
    f = pkg._L().ds3_gemm_tail_share_steps

    def pieces(tail, kb, q):
        return max(((t + 1) * kb - 1) // q - (t * kb) // q + 1 for t in range(tail))

    for wgs in (8, 32, 64):
        for tail in range(1, wgs):
            for kb in (1, 2, 3, 4, 7, 12, 16, 32, 56, 57, 144):
                q = f(tail, kb, wgs)
                q0 = -(-tail * kb // wgs)
                if q == 0:                       # nothing below a whole tile qualifies
                    assert all(pieces(tail, kb, c) > 2 for c in range(q0, kb)), (tail, kb, wgs)
                    continue
                assert q0 <= q < kb and -(-tail * kb // q) <= wgs, (tail, kb, wgs, q)
                assert pieces(tail, kb, q) <= 2, (tail, kb, wgs, q)
                assert all(pieces(tail, kb, c) > 2 for c in range(q0, q)), (tail, kb, wgs, q)
    assert f(16, 56, 32) == 28 and f(24, 144, 32) == 108 and f(12, 56, 32) == 28
    assert f(0, 56, 32) == 0 and f(40, 56, 32) == 0


def test_later_entry_points_reject_bad_arguments_on_the_host(pkg):
    L = pkg._L()
    buf = (ctypes.c_uint8 * 4096)()
    p = (ctypes.addressof(buf) + 15) & ~15
    # power-of-two forms share the checks of the plain calls
    assert L.ds3_quant_act_1x128_pow2(None, 1, 4, 128, 128, p, 128, p, 1, 4, None) == 1
    assert L.ds3_gemm_fp8_bs_pow2(-1, 16, 16, 100, p, 128, p, 1, 16, p, 128, p, 1, 1, 0, p, 1, 16, 0, None, 0, None) == 2
    assert L.ds3_gemm_fp8_bs_pow2(7, 16, 16, 128, p, 128, p, 1, 16, p, 128, p, 1, 1, 0, p, 1, 16, 0, None, 0, None) == 5
    assert L.ds3_grouped_gemm_fp8_bs_pow2(-1, 1, None, 16, 16, 128, p, 128, p, 1, 16, p, 128, p, p, 1, 16, None, 0, None) == 1
    # dual-layout weight quantizer
    d = L.ds3_quant_w_128x128_dual
    assert d(p, 1, 16, 128, 128, p, 128, p, None, 16, p, None) == 1           # q_t missing
    assert d(p, 1, 16, 128, 128, p, 128, p, p, 8, p, None) == 2               # ldqt < n
    assert d(p, 1, 20, 128, 128, p, 128, p, p, 24, p, None) == 3              # ldqt % 16
    assert d(p, 1, 0, 128, 128, None, 128, None, None, 0, None, None) == 0    # empty
    # cache re-tiling
    r = L.ds3_retile_1x128_to_128x1
    assert r(p, 16, 128, 128, None, 1, 16, p, 16, p, 1, 128, None) == 1
    assert r(p, 16, 136, 144, p, 1, 16, p, 16, p, 1, 136, None) == 3          # cols % 16
    assert r(p, 16, 128, 64, p, 1, 16, p, 16, p, 1, 128, None) == 2           # ldq < cols
    assert r(p, 20, 128, 128, p, 1, 20, p, 16, p, 1, 128, None) == 2          # ldqt < rows
    assert r(p, -1, 128, 128, p, 1, 16, p, 16, p, 1, 128, None) == 2
    # fused producers
    sq = L.ds3_swiglu_quant_1x128
    assert sq(p, 4, 12, 24, p, 16, p, 1, 4, None) == 3                        # inter % 8
    assert sq(p, 4, 16, 24, p, 16, p, 1, 4, None) == 2                        # ldh < 2 * inter
    assert sq(p, 4, 16, 32, None, 16, p, 1, 4, None) == 1
    for gq in (L.ds3_grouped_gemm_swiglu_quant_fp8_bs, L.ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2):
        ok = (2, p, 32, 128, 128, p, 128, p, 1, 32, p, 128, p, p, 128, p, 1, 32, None, 0, None)

        def with_(i, v):
            return ok[:i] + (v,) + ok[i + 1:]
        assert gq(*with_(3, 64)) == 2                                         # inter % 128
        assert gq(*with_(4, 100)) == 2                                        # K % 128
        assert gq(*with_(4, 0)) == 2                                          # K == 0
        assert gq(*with_(14, 64)) == 2                                        # ldq < inter
        assert gq(*with_(14, 136)) == 3                                       # ldq % 16
        assert gq(*with_(13, None)) == 1 and gq(*with_(15, None)) == 1        # outputs missing
        assert gq(*with_(1, None)) == 1 and gq(*with_(10, None)) == 1         # offsets, weight missing
        assert gq(*with_(0, 0)) == 0 and gq(*with_(2, 0)) == 0                # nothing to do
        assert gq(*with_(0, -1)) == 2 and gq(*with_(0, 1024)) == 5
    rn = L.ds3_rmsnorm_quant_1x128
    assert rn(p, 4, 128, 128, None, 1e-6, None, 0, p, 128, p, 1, 4, None) == 1      # gamma missing
    assert rn(p, 4, 8200, 8200, p, 1e-6, None, 0, p, 8208, p, 1, 4, None) == 5      # row longer than 8192
    assert rn(p, 4, 128, 128, p, -1.0, None, 0, p, 128, p, 1, 4, None) == 2         # negative eps
    assert rn(p, 4, 128, 128, p, 1e-6, p, 64, p, 128, p, 1, 4, None) == 2           # ldy < cols
    # optimizer
    ad = L.ds3_adamw_bf16_states
    assert ad(16, p, p, p, p, None, 1e-3, 0.9, 0.95, 1e-8, 0.1, 0, None) == 2       # steps count from 1
    assert ad(12, p, p, p, p, None, 1e-3, 0.9, 0.95, 1e-8, 0.1, 1, None) == 3       # n % 8
    assert ad(16, p, p, p, p, None, 1e-3, 1.0, 0.95, 1e-8, 0.1, 1, None) == 2       # beta1 == 1
    assert ad(16, None, p, p, p, None, 1e-3, 0.9, 0.95, 1e-8, 0.1, 1, None) == 1
    assert ad(0, None, None, None, None, None, 1e-3, 0.9, 0.95, 1e-8, 0.1, 1, None) == 0
    # probes
    assert L.ds3_probe_mfma_fp8(10, 4, None, None) == 1
    assert L.ds3_probe_lds_feed(p, 1 << 20, 100, 10, 4, p, None) == 2               # row stride not a multiple of 128
    assert L.ds3_probe_lds_feed(p, 1 << 20, 7168, 10, 4, p, None) == 5              # window smaller than 4096 rows
