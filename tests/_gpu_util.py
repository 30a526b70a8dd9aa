"""Helpers for the GPU parity tests: host<->device marshalling only."""
import numpy as np
import torch

DEV = "cuda:0"


def dev(x: np.ndarray, bf16: bool = False) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.to(torch.bfloat16) if bf16 else t


def host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().contiguous().numpy()


def normwise(got: np.ndarray, want: np.ndarray) -> float:
    got = got.astype(np.float64)
    den = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / den) if den > 0 else float(np.linalg.norm(got))


def announce(msg: str):
    print(f"[case] {msg}", flush=True)


# The matrix unit's 128-term sum is good to about 13 bits below the sum of the magnitudes
# (tests/test_gpu_mfma_accumulation.py measures 2^-12.6 and asserts 2^-11.6).
ACC_BETA = 2.0 ** -11.6


def magnitude_sum(a, sa, b, sb, sb_per_row: bool = False) -> np.ndarray:
    """sum_k |a_mk sa| |b_nk sb| in FP64: what the accumulation error of an output is bounded by."""
    from oracle import ds3_oracle as orc
    ad = np.abs(orc.dequant_rows(a, sa))
    bd = np.abs(orc.dequant_rows(b, sb) if sb_per_row else orc.dequant_blocks(b, sb))
    return ad @ bd.T


def bf16_elementwise(got: np.ndarray, want64: np.ndarray, mag: np.ndarray):
    """Element-wise view of a BF16 result against the unrounded FP64 reference.  The kernel rounds
    an FP32 sum v to BF16 with |v - reference| <= ACC_BETA * mag, so every output must satisfy
        |got - reference| <= ulp_bf16 / 2 + ACC_BETA * mag.
    Returns (the largest value of (|got - reference| - ACC_BETA * mag) / ulp_bf16, which must not
    exceed 0.5; the fraction of outputs that equal round_to_bf16(reference) exactly)."""
    w32 = np.ascontiguousarray(want64, dtype=np.float32)
    u = w32.view(np.uint32).astype(np.uint64)
    rb = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32).view(np.float32).astype(np.float64)
    g = got.astype(np.float64)
    big = np.maximum(np.maximum(np.abs(rb), np.abs(g)), 2.0 ** -126)
    ulp = 2.0 ** (np.floor(np.log2(big)) - 7)
    excess = (np.abs(g - want64) - ACC_BETA * mag) / ulp
    return float(excess.max()), float(np.mean(g == rb))
