"""Seeded generators for the five synthetic workloads.

Shapes follow the model hyper-parameters of Section 4.2 of the DeepSeek-V3
report (hidden 7168, expert intermediate 2048, 256 routed experts, top-8,
MLA ranks 1536 / 512, 128 heads); the dense-FFN width 18432 comes from the
benchmark definition.  All tensors are returned as float32 numpy arrays; the
"BF16" ones hold only BF16-representable values so that the widening to
float32 is exact on both sides of a comparison.
"""
from __future__ import annotations

import numpy as np

HIDDEN = 7168
DENSE_INTER = 18432
MOE_INTER = 2048
N_ROUTED = 256
TOP_K = 8
LOCAL_EXPERTS = 32
Q_LORA, KV_LORA, ROPE_DIM, N_HEADS = 1536, 512, 64, 128


def seed_for(config: int, tensor: int) -> int:
    return 1000 * config + tensor


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest BF16 value (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of a float32 array that holds BF16-representable values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "not BF16-representable"
    return (u >> 16).astype(np.uint16).reshape(x.shape)


def normal(shape, std, seed, bf16=True) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return bf16_round(x) if bf16 else x


# ---- config 1: tiny dense Fprop, FP32 inputs with entry outliers ------------
def cfg1(m=256, n=512, k=1024):
    out = []
    for idx, shape in enumerate([(m, k), (n, k)]):
        rng = np.random.default_rng(seed_for(1, idx))
        x = rng.standard_normal(shape, dtype=np.float32)
        mask = rng.random(shape) < 1e-3               # 0.1% of entries are x100 outliers
        x[mask] *= np.float32(100.0)
        out.append(x)
    return out[0], out[1]


# ---- config 2: dense FFN up-projection --------------------------------------
def cfg2_x(m=4096, k=HIDDEN):
    """Activations ~N(0,1) with 1% of the channels (columns) scaled x50."""
    rng = np.random.default_rng(seed_for(2, 0))
    x = rng.standard_normal((m, k), dtype=np.float32)
    cols = rng.choice(k, size=max(1, k // 100), replace=False)
    x[:, cols] *= np.float32(50.0)
    return bf16_round(x)


def cfg2_w(n=DENSE_INTER, k=HIDDEN):
    return normal((n, k), 0.02, seed_for(2, 1))


# ---- config 3: one GPU's share of the MoE experts ---------------------------
def cfg3_routing(tokens=8192, n_experts=N_ROUTED, top_k=TOP_K, local=LOCAL_EXPERTS, sigma_b=0.02, experts=None):
    """Top-k routing on sigmoid affinities plus a per-expert bias (Section 2.1.2,
    auxiliary-loss-free balancing: the bias enters the top-k selection only).
    Returns (group_sizes[local], group_offsets[local+1], token_ids) where
    token_ids lists, expert by expert, the tokens routed to experts 0..local-1
    (or to the experts listed in `experts`).  Ties go to the lower expert index
    (stable sort)."""
    rng = np.random.default_rng(seed_for(3, 0))
    logits = rng.standard_normal((tokens, n_experts))
    bias = rng.standard_normal(n_experts) * sigma_b
    score = 1.0 / (1.0 + np.exp(-logits)) + bias
    order = np.argsort(-score, axis=1, kind="stable")[:, :top_k]
    held = list(range(local)) if experts is None else [int(e) for e in experts]
    sizes = np.zeros(len(held), dtype=np.int64)
    ids = []
    for i, e in enumerate(held):
        tok = np.nonzero((order == e).any(axis=1))[0]
        sizes[i] = tok.size
        ids.append(tok)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    return sizes, offsets, np.concatenate(ids) if ids else np.zeros(0, np.int64)


def cfg3_stress_experts(local=LOCAL_EXPERTS, sigma_b=0.05):
    """The stress variant of config 3: with a wider bias distribution the per-expert load runs from
    0 to about 4x the mean; the GPU is given the local/2 least and the local/2 most loaded experts
    (in index order), so that empty and very large groups meet in one call."""
    sizes, _, _ = cfg3_routing(local=N_ROUTED, sigma_b=sigma_b)
    order = np.argsort(sizes, kind="stable")
    return sorted(int(e) for e in np.concatenate([order[:local // 2], order[-(local // 2):]]))


def cfg3_tokens(total_rows, k=HIDDEN):
    return normal((total_rows, k), 1.0, seed_for(3, 1))


def _expert_weight(tensor, e, shape):
    """One expert's weight ~N(0, 0.02), BF16-representable; every expert has a random stream of its
    own (seed sequence [seed_for(3, tensor), e]), so any subset can be drawn without the others."""
    rng = np.random.default_rng([seed_for(3, tensor), int(e)])
    return bf16_round(rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02))


def cfg3_w13_expert(e, inter=MOE_INTER, k=HIDDEN):
    """Fused gate|up weight of expert e: [2*inter][k]; rows 0..inter-1 gate, rest up."""
    return _expert_weight(2, e, (2 * inter, k))


def cfg3_w2_expert(e, inter=MOE_INTER, k=HIDDEN):
    """Down-projection weight of expert e: [k][inter]."""
    return _expert_weight(3, e, (k, inter))


def cfg3_w13(g=LOCAL_EXPERTS, inter=MOE_INTER, k=HIDDEN):
    """Fused gate|up weights of experts 0..g-1: [g][2*inter][k]."""
    return np.stack([cfg3_w13_expert(e, inter, k) for e in range(g)])


def cfg3_w2(g=LOCAL_EXPERTS, inter=MOE_INTER, k=HIDDEN):
    return np.stack([cfg3_w2_expert(e, inter, k) for e in range(g)])


# ---- config 4: backward of the config-2 layer -------------------------------
def interleave_gate_up(t: np.ndarray, block: int = 128) -> np.ndarray:
    """Row order of the fused gate|up weight for the GEMM whose epilogue applies SwiGLU:
    [..., 2*I, ...] with gate rows [0, I) and up rows [I, 2I) on axis -2 becomes
    gate block 0, up block 0, gate block 1, up block 1, ... in blocks of `block` rows.
    Used with block = 128 on the codes and block = 1 on their 128x128 scales."""
    two_i = t.shape[-2]
    nb = two_i // 2 // block
    assert two_i == 2 * nb * block
    lead, tail = t.shape[:-2], t.shape[-1:]
    v = t.reshape(*lead, 2, nb, block, *tail)
    return np.ascontiguousarray(np.swapaxes(v, -4, -3)).reshape(t.shape)


def cfg4_dy(m=4096, n=DENSE_INTER):
    return normal((m, n), 1e-2, seed_for(4, 0))


# ---- config 5: MLA projections ----------------------------------------------
def cfg5_shapes(tokens=8192):
    """(name, M, N, K) of the four projections of Section 2.1.1."""
    return [
        ("q_a", tokens, Q_LORA, HIDDEN),
        ("kv_a", tokens, KV_LORA + ROPE_DIM, HIDDEN),
        ("q_b", tokens, N_HEADS * (128 + ROPE_DIM), Q_LORA),
        ("kv_b", tokens, N_HEADS * (128 + 128), KV_LORA),
    ]


def cfg5_act(m, k, idx):
    return normal((m, k), 1.0, seed_for(5, idx))


def cfg5_w(n, k, idx):
    return normal((n, k), 0.02, seed_for(5, 10 + idx))
