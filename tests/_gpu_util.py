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
