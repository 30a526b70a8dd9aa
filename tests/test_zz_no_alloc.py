"""The GEMM entry point that allocates nothing (its partial sums go through a statically
allocated device array of the library) against the entry point that takes the caller's
workspace: same kernels, same sharing of tiles, so the outputs are equal bit for bit -- on two
calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from oracle import ds3_oracle as orc
from tests._gpu_util import announce, dev, host, normwise

pytestmark = pytest.mark.gpu


def _rand_codes(rng, shape):
    c = rng.integers(0, 0x7F, size=shape).astype(np.uint8)
    return c | (rng.integers(0, 2, size=shape) << 7).astype(np.uint8)


def test_no_alloc_entry_point_matches_the_workspace_entry_point(ds3):
    rng = np.random.default_rng(91)
    for (m, n, k) in [(2048, 1536, 2048), (384, 640, 1024)]:        # both share tail tiles along K
        announce(f"no-alloc GEMM {m}x{n}x{k}")
        assert ds3.ds3_gemm_workspace_bytes(m, n, k) > 0
        a, b = _rand_codes(rng, (m, k)), _rand_codes(rng, (n, k))
        sa = np.exp(rng.standard_normal((m, k // 128))).astype(np.float32)
        sb = np.exp(rng.standard_normal(((n + 127) // 128, k // 128))).astype(np.float32)
        ad, sad, bd, sbd = dev(a), dev(sa), dev(b), dev(sb)
        for dt, tol in ((torch.bfloat16, 2e-3), (torch.float32, 1e-4)):
            want = ds3.ds3_gemm_fp8_bs(ad, sad, bd, sbd, out_dtype=dt)       # caller's workspace (from the binding's cache)
            got = torch.full((m, n), 3.0, dtype=dt, device="cuda:0")
            ds3.ds3_gemm_fp8_bs_noalloc(ad, sad, bd, sbd, got)
            assert torch.equal(got, want), (m, n, k, dt)
            assert normwise(host(got), orc.gemm_fp8_bs(a, sa, b, sb)) <= tol
        # accumulation into FP32, and a second call right behind the first on the same array
        acc = torch.zeros((m, n), dtype=torch.float32, device="cuda:0")
        ds3.ds3_gemm_fp8_bs_noalloc(ad, sad, bd, sbd, acc, accumulate=True)
        ds3.ds3_gemm_fp8_bs_noalloc(ad, sad, bd, sbd, acc, accumulate=True)
        once = ds3.ds3_gemm_fp8_bs(ad, sad, bd, sbd, out_dtype=torch.float32)
        assert torch.equal(acc, 2 * once)
