"""Python binding of libds3: the fine-grained FP8 linear layer of DeepSeek-V3
(Section 3.3) as hand-written HIP kernels for MI355X (gfx950).

The functions here have the names of the C entry points declared in
include/ds3.h and only marshal arguments: torch tensors supply device memory
and the current stream, every step of the path runs in the library's kernels.
There is no CPU fallback: importing this package without a built libds3.so
raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libds3.so")

DS3_OK = 0
DS3_F32, DS3_BF16 = 0, 1
DS3_BSCALE_128x128, DS3_BSCALE_PER_ROW = 0, 1

SYMBOLS = [
    "ds3_quant_act_1x128", "ds3_quant_act_128x1", "ds3_quant_w_128x128",
    "ds3_gemm_fp8_bs", "ds3_grouped_gemm_fp8_bs", "ds3_gemm_fp8_bs_v", "ds3_grouped_gemm_fp8_bs_v",
    "ds3_gemm_num_variants", "ds3_gemm_workspace_bytes", "ds3_gemm_workspace_bytes_v", "ds3_gemm_tail_share_steps", "ds3_gemm_workspace_init", "ds3_gemm_fp8_bs_noalloc", "ds3_gemm_noalloc_scratch_bytes", "ds3_swiglu", "ds3_status_string",
    "ds3_quant_act_1x128_pow2", "ds3_quant_act_128x1_pow2", "ds3_quant_w_128x128_pow2",
    "ds3_gemm_fp8_bs_pow2", "ds3_grouped_gemm_fp8_bs_pow2",
    "ds3_probe_mfma_fp8", "ds3_probe_lds_feed", "ds3_swiglu_quant_1x128", "ds3_swiglu_quant_1x128_pow2",
    "ds3_retile_1x128_to_128x1", "ds3_retile_1x128_to_128x1_pow2",
    "ds3_quant_w_128x128_dual", "ds3_quant_w_128x128_dual_pow2",
    "ds3_rmsnorm_quant_1x128", "ds3_rmsnorm_quant_1x128_pow2", "ds3_adamw_bf16_states",
    "ds3_quant_act_1x128_e5m6", "ds3_dequant_e5m6",
    "ds3_grouped_gemm_swiglu_quant_fp8_bs", "ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2",
    "ds3_grouped_gemm_workspace_bytes",
]


class Ds3Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2412_19437_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    for sfx in ("", "_pow2"):
        getattr(lib, "ds3_quant_act_1x128" + sfx).argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, i64, i64, vp]
        getattr(lib, "ds3_quant_act_128x1" + sfx).argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, i64, i64, vp]
        getattr(lib, "ds3_quant_w_128x128" + sfx).argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, vp]
    gemm = [i64, i64, i64, vp, i64, vp, i64, i64, vp, i64, vp, i64, i64, i32, vp, i32, i64, i32, vp, sz, vp]
    lib.ds3_gemm_fp8_bs.argtypes = gemm
    lib.ds3_gemm_fp8_bs_v.argtypes = [i32] + gemm
    lib.ds3_gemm_fp8_bs_pow2.argtypes = [i32] + gemm
    lib.ds3_gemm_fp8_bs_noalloc.argtypes = gemm[:-3] + [vp]
    lib.ds3_gemm_noalloc_scratch_bytes.argtypes = []
    lib.ds3_gemm_noalloc_scratch_bytes.restype = sz
    grouped = [i32, vp, i64, i64, i64, vp, i64, vp, i64, i64, vp, i64, vp, vp, i32, i64, vp, sz, vp]
    lib.ds3_grouped_gemm_fp8_bs.argtypes = grouped
    lib.ds3_grouped_gemm_fp8_bs_v.argtypes = [i32] + grouped
    lib.ds3_grouped_gemm_fp8_bs_pow2.argtypes = [i32] + grouped
    lib.ds3_swiglu.argtypes = [vp, i64, i64, i64, vp, i64, vp]
    lib.ds3_swiglu_quant_1x128.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, i64, vp]
    for name in ("ds3_grouped_gemm_swiglu_quant_fp8_bs", "ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2"):
        getattr(lib, name).argtypes = [ctypes.c_int32, vp, i64, i64, i64, vp, i64, vp, i64, i64, vp, i64, vp, vp, i64, vp, i64, i64,
                                       vp, ctypes.c_size_t, vp]
    lib.ds3_grouped_gemm_workspace_bytes.argtypes = []
    lib.ds3_grouped_gemm_workspace_bytes.restype = ctypes.c_size_t
    lib.ds3_swiglu_quant_1x128_pow2.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, i64, vp]
    lib.ds3_retile_1x128_to_128x1.argtypes = [vp, i64, i64, i64, vp, i64, i64, vp, i64, vp, i64, i64, vp]
    lib.ds3_retile_1x128_to_128x1_pow2.argtypes = [vp, i64, i64, i64, vp, i64, i64, vp, i64, vp, i64, i64, vp]
    lib.ds3_quant_w_128x128_dual.argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, vp, i64, vp, vp]
    lib.ds3_quant_w_128x128_dual_pow2.argtypes = [vp, i32, i64, i64, i64, vp, i64, vp, vp, i64, vp, vp]
    f32 = ctypes.c_float
    lib.ds3_rmsnorm_quant_1x128.argtypes = [vp, i64, i64, i64, vp, f32, vp, i64, vp, i64, vp, i64, i64, vp]
    lib.ds3_rmsnorm_quant_1x128_pow2.argtypes = [vp, i64, i64, i64, vp, f32, vp, i64, vp, i64, vp, i64, i64, vp]
    lib.ds3_quant_act_1x128_e5m6.argtypes = [vp, i64, i64, i64, vp, i64, vp, i64, i64, vp]
    lib.ds3_dequant_e5m6.argtypes = [vp, i64, i64, i64, vp, i64, i64, vp, i64, vp]
    lib.ds3_adamw_bf16_states.argtypes = [i64, vp, vp, vp, vp, vp, f32, f32, f32, f32, f32, i64, vp]
    lib.ds3_probe_mfma_fp8.argtypes = [i32, i32, vp, vp]
    lib.ds3_probe_lds_feed.argtypes = [vp, sz, i64, i32, i32, vp, vp]
    lib.ds3_gemm_num_variants.argtypes = []
    lib.ds3_gemm_workspace_bytes.argtypes = [i64, i64, i64]
    lib.ds3_gemm_workspace_bytes.restype = sz
    lib.ds3_gemm_workspace_bytes_v.argtypes = [i32, i64, i64, i64, i32]
    lib.ds3_gemm_workspace_bytes_v.restype = sz
    lib.ds3_gemm_tail_share_steps.argtypes = [i32, i32, i32]
    lib.ds3_gemm_workspace_init.argtypes = [vp, sz, vp]
    lib.ds3_gemm_tail_share_steps.restype = i32
    lib.ds3_status_string.argtypes = [i32]
    lib.ds3_status_string.restype = ctypes.c_char_p
    for name in SYMBOLS:
        getattr(lib, name)
    return lib


_lib = None


def _L() -> ctypes.CDLL:
    """The loaded library (loaded on first use, so that the build module can be
    imported before the library exists); raises if it has not been built."""
    global _lib
    if _lib is None:
        _lib = _load()
    return _lib


def status_string(status: int) -> str:
    return _L().ds3_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != DS3_OK:
        raise Ds3Error(status, where)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DS3_F32
    if t.dtype == torch.bfloat16:
        return DS3_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _rows2d(t: torch.Tensor, name: str):
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with contiguous rows")
    return t.shape[0], t.shape[1], t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))


def _codes(rows: int, cols: int, device) -> torch.Tensor:
    """uint8 [rows][cols] whose leading dimension is padded to a multiple of 16."""
    ld = (cols + 15) // 16 * 16
    return torch.empty((rows, ld), dtype=torch.uint8, device=device)[:, :cols]


def _out(rows: int, cols: int, dtype, device) -> torch.Tensor:
    """GEMM output [rows][cols] whose leading dimension is padded to a multiple of 8 elements."""
    ld = (cols + 7) // 8 * 8
    return torch.empty((rows, ld), dtype=dtype, device=device)[:, :cols]


def _scales(rows: int, blocks: int, device, k_major: bool) -> torch.Tensor:
    """Logical [rows][blocks] FP32 tensor; k_major stores it as [blocks][rows]."""
    if k_major:
        return torch.empty((blocks, rows), dtype=torch.float32, device=device).t()
    return torch.empty((rows, blocks), dtype=torch.float32, device=device)


def _quant_act_1x128(entry: str, x: torch.Tensor, k_major_scales: bool):
    m, k, ldx = _rows2d(x, "x")
    q = _codes(m, k, x.device)
    s = _scales(m, (k + 127) // 128, x.device, k_major_scales)
    st = getattr(_L(), entry)(x.data_ptr(), _dt(x), m, k, ldx, q.data_ptr(), (k + 15) // 16 * 16,
                              s.data_ptr(), s.stride(0), s.stride(1), _stream())
    _check(st, entry)
    return q, s


def _quant_act_128x1(entry: str, x: torch.Tensor, k_major_scales: bool):
    t, c, ldx = _rows2d(x, "x")
    ldq = (t + 15) // 16 * 16
    q_t = _codes(c, t, x.device)
    s_t = _scales(c, (t + 127) // 128, x.device, k_major_scales)
    st = getattr(_L(), entry)(x.data_ptr(), _dt(x), t, c, ldx, q_t.data_ptr(), ldq,
                              s_t.data_ptr(), s_t.stride(0), s_t.stride(1), _stream())
    _check(st, entry)
    return q_t, s_t


def _quant_w_128x128(entry: str, w: torch.Tensor):
    n, k, ldw = _rows2d(w, "w")
    q = _codes(n, k, w.device)
    s = torch.empty(((n + 127) // 128, (k + 127) // 128), dtype=torch.float32, device=w.device)
    st = getattr(_L(), entry)(w.data_ptr(), _dt(w), n, k, ldw, q.data_ptr(), (k + 15) // 16 * 16, s.data_ptr(),
                              _stream())
    _check(st, entry)
    return q, s


def ds3_quant_act_1x128(x: torch.Tensor, k_major_scales: bool = True):
    """x [M][K] FP32/BF16 -> (codes uint8 [M][K], scales FP32 logical [M][ceil(K/128)])."""
    return _quant_act_1x128("ds3_quant_act_1x128", x, k_major_scales)


def ds3_quant_act_1x128_pow2(x: torch.Tensor, k_major_scales: bool = True):
    """As ds3_quant_act_1x128 with power-of-two scales."""
    return _quant_act_1x128("ds3_quant_act_1x128_pow2", x, k_major_scales)


def ds3_quant_act_128x1(x: torch.Tensor, k_major_scales: bool = True):
    """x [T][C] -> (codes uint8 [C][T] token-contiguous, scales logical [C][ceil(T/128)])."""
    return _quant_act_128x1("ds3_quant_act_128x1", x, k_major_scales)


def ds3_quant_act_128x1_pow2(x: torch.Tensor, k_major_scales: bool = True):
    """As ds3_quant_act_128x1 with power-of-two scales."""
    return _quant_act_128x1("ds3_quant_act_128x1_pow2", x, k_major_scales)


def ds3_quant_w_128x128(w: torch.Tensor):
    """w [N][K] -> (codes uint8 [N][K], scales FP32 [ceil(N/128)][ceil(K/128)])."""
    return _quant_w_128x128("ds3_quant_w_128x128", w)


def ds3_quant_w_128x128_pow2(w: torch.Tensor):
    """As ds3_quant_w_128x128 with power-of-two scales."""
    return _quant_w_128x128("ds3_quant_w_128x128_pow2", w)


def ds3_gemm_fp8_bs(a, sa, b, sb, sb_mode: int = DS3_BSCALE_128x128, out_dtype=torch.bfloat16,
                    c: torch.Tensor | None = None, accumulate: bool = False, variant: int = -1, workspace="auto"):
    """C[M][N] (+)= block-scaled product of codes a [M][K] (scales sa, logical
    [M][K/128]) and b [N][K] (scales sb: [ceil(N/128)][K/128], or [N][K/128]
    when sb_mode is DS3_BSCALE_PER_ROW).  workspace: "auto" (a cached tensor of the
    size the library asks for), None (never share tiles along K) or a uint8 tensor."""
    return _gemm("ds3_gemm_fp8_bs_v", a, sa, b, sb, sb_mode, out_dtype, c, accumulate, variant, workspace)


def ds3_gemm_fp8_bs_pow2(a, sa, b, sb, sb_mode: int = DS3_BSCALE_128x128, out_dtype=torch.bfloat16,
                         c: torch.Tensor | None = None, accumulate: bool = False, variant: int = -1, workspace="auto"):
    """As ds3_gemm_fp8_bs for operands whose scales are all powers of two."""
    return _gemm("ds3_gemm_fp8_bs_pow2", a, sa, b, sb, sb_mode, out_dtype, c, accumulate, variant, workspace)


_workspaces: dict = {}


def gemm_workspace(nbytes: int, device) -> torch.Tensor | None:
    """A per-device, per-stream uint8 tensor of at least nbytes (None for 0), kept for reuse:
    the GEMM's workspace must not be shared by calls that may overlap."""
    if nbytes <= 0:
        return None
    key = (torch.device(device).index or 0, _stream())
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        ws = new_gemm_workspace(nbytes, device)
        _workspaces[key] = ws
    return ws


def new_gemm_workspace(nbytes: int, device) -> torch.Tensor:
    """A uint8 tensor of nbytes, prepared with ds3_gemm_workspace_init on the current stream."""
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    _check(_L().ds3_gemm_workspace_init(ws.data_ptr(), nbytes, _stream()), "ds3_gemm_workspace_init")
    return ws


def _gemm(entry, a, sa, b, sb, sb_mode, out_dtype, c, accumulate, variant, workspace="auto"):
    m, k, lda = _rows2d(a, "a")
    n, kb_, ldb = _rows2d(b, "b")
    if kb_ != k:
        raise ValueError("a and b disagree on K")
    if c is None:
        c = _out(m, n, out_dtype, a.device)
    _, _, ldc = _rows2d(c, "c")
    if isinstance(workspace, str):                 # "auto": what the library asks for, from the cache
        workspace = gemm_workspace(_L().ds3_gemm_workspace_bytes_v(variant, m, n, k, sb_mode), a.device)
    st = getattr(_L(), entry)(variant, m, n, k, a.data_ptr(), lda, sa.data_ptr(), sa.stride(0), sa.stride(1),
                              b.data_ptr(), ldb, sb.data_ptr(), sb.stride(0), sb.stride(1), sb_mode,
                              c.data_ptr(), _dt(c), ldc, int(accumulate),
                              workspace.data_ptr() if workspace is not None else None,
                              workspace.numel() if workspace is not None else 0, _stream())
    _check(st, entry)
    return c


def ds3_grouped_gemm_fp8_bs(a, sa, group_offsets, b, sb, out_dtype=torch.bfloat16,
                            c: torch.Tensor | None = None, variant: int = -1, workspace="auto"):
    """Per expert g: rows [off[g], off[g+1]) of a times b[g] ([G][N][K] codes,
    sb [G][ceil(N/128)][K/128]).  group_offsets: int32 device tensor of G+1.
    workspace: "auto" (the cached one: tiles are handed out through a queue), None (static walk)
    or a prepared uint8 tensor; the result is the same bit for bit."""
    return _grouped("ds3_grouped_gemm_fp8_bs_v", a, sa, group_offsets, b, sb, out_dtype, c, variant, workspace)


def ds3_grouped_gemm_fp8_bs_pow2(a, sa, group_offsets, b, sb, out_dtype=torch.bfloat16,
                                 c: torch.Tensor | None = None, variant: int = -1, workspace="auto"):
    """As ds3_grouped_gemm_fp8_bs for operands whose scales are all powers of two."""
    return _grouped("ds3_grouped_gemm_fp8_bs_pow2", a, sa, group_offsets, b, sb, out_dtype, c, variant, workspace)


def _grouped_ws(workspace, device):
    if isinstance(workspace, str):
        workspace = gemm_workspace(_L().ds3_grouped_gemm_workspace_bytes(), device)
    return (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)


def _grouped(entry, a, sa, group_offsets, b, sb, out_dtype, c, variant, workspace="auto"):
    m, k, lda = _rows2d(a, "a")
    g, n, kk = b.shape
    if kk != k or not b.is_contiguous() or not sb.is_contiguous():
        raise ValueError("b must be contiguous [G][N][K] and sb contiguous")
    if group_offsets.dtype != torch.int32 or group_offsets.numel() != g + 1:
        raise ValueError("group_offsets must be int32 of length G+1")
    if c is None:
        c = _out(m, n, out_dtype, a.device)
    _, _, ldc = _rows2d(c, "c")
    st = getattr(_L(), entry)(variant, g, group_offsets.data_ptr(), m, n, k, a.data_ptr(), lda,
                              sa.data_ptr(), sa.stride(0), sa.stride(1), b.data_ptr(), k, sb.data_ptr(),
                              c.data_ptr(), _dt(c), ldc, *_grouped_ws(workspace, a.device), _stream())
    _check(st, entry)
    return c


def ds3_swiglu(h: torch.Tensor):
    """h [rows][2*inter] BF16 (gate | up) -> silu(gate) * up, BF16 [rows][inter]."""
    rows, two_i, ldh = _rows2d(h, "h")
    if h.dtype != torch.bfloat16 or two_i % 2:
        raise TypeError("h must be BF16 with an even number of columns")
    out = torch.empty((rows, two_i // 2), dtype=torch.bfloat16, device=h.device)
    st = _L().ds3_swiglu(h.data_ptr(), rows, two_i // 2, ldh, out.data_ptr(), two_i // 2, _stream())
    _check(st, "ds3_swiglu")
    return out


def _quant_w_dual(entry: str, w: torch.Tensor):
    n, k, ldw = _rows2d(w, "w")
    q, q_t = _codes(n, k, w.device), _codes(k, n, w.device)
    nb, kb = (n + 127) // 128, (k + 127) // 128
    s = torch.empty((nb, kb), dtype=torch.float32, device=w.device)
    s_t = torch.empty((kb, nb), dtype=torch.float32, device=w.device)
    st = getattr(_L(), entry)(w.data_ptr(), _dt(w), n, k, ldw, q.data_ptr(), (k + 15) // 16 * 16, s.data_ptr(),
                              q_t.data_ptr(), (n + 15) // 16 * 16, s_t.data_ptr(), _stream())
    _check(st, entry)
    return q, s, q_t, s_t


def ds3_quant_w_128x128_dual(w: torch.Tensor):
    """w [N][K] -> (codes [N][K], scales [N/128][K/128], codes of the transpose [K][N], its scales [K/128][N/128])."""
    return _quant_w_dual("ds3_quant_w_128x128_dual", w)


def ds3_quant_w_128x128_dual_pow2(w: torch.Tensor):
    """As ds3_quant_w_128x128_dual with power-of-two scales."""
    return _quant_w_dual("ds3_quant_w_128x128_dual_pow2", w)


def _rmsnorm_quant(entry: str, x, gamma, eps, want_y, k_major_scales):
    rows, cols, ldx = _rows2d(x, "x")
    if x.dtype != torch.bfloat16 or gamma.dtype != torch.float32 or gamma.numel() != cols or not gamma.is_contiguous():
        raise TypeError("x must be BF16 and gamma a contiguous FP32 vector of x's width")
    q = _codes(rows, cols, x.device)
    s = _scales(rows, (cols + 127) // 128, x.device, k_major_scales)
    y = torch.empty((rows, cols), dtype=torch.bfloat16, device=x.device) if want_y else None
    st = getattr(_L(), entry)(x.data_ptr(), rows, cols, ldx, gamma.data_ptr(), float(eps),
                              y.data_ptr() if want_y else None, cols, q.data_ptr(), (cols + 15) // 16 * 16,
                              s.data_ptr(), s.stride(0), s.stride(1), _stream())
    _check(st, entry)
    return (q, s, y) if want_y else (q, s)


def ds3_rmsnorm_quant_1x128(x, gamma, eps: float = 1e-6, want_y: bool = False, k_major_scales: bool = True):
    """RMSNorm(x) * gamma rounded to BF16, 1x128-quantized: (codes, scales[, the BF16 activation])."""
    return _rmsnorm_quant("ds3_rmsnorm_quant_1x128", x, gamma, eps, want_y, k_major_scales)


def ds3_rmsnorm_quant_1x128_pow2(x, gamma, eps: float = 1e-6, want_y: bool = False, k_major_scales: bool = True):
    """As ds3_rmsnorm_quant_1x128 with power-of-two scales."""
    return _rmsnorm_quant("ds3_rmsnorm_quant_1x128_pow2", x, gamma, eps, want_y, k_major_scales)


def ds3_quant_act_1x128_e5m6(x: torch.Tensor, k_major_scales: bool = True):
    """x [M][K] BF16 -> (packed E5M6 codes uint8 [M][3K/2], power-of-two scales logical [M][ceil(K/128)])."""
    m, k, ldx = _rows2d(x, "x")
    if x.dtype != torch.bfloat16:
        raise TypeError("x must be BF16")
    q = torch.empty((m, k * 3 // 2), dtype=torch.uint8, device=x.device)
    s = _scales(m, (k + 127) // 128, x.device, k_major_scales)
    st = _L().ds3_quant_act_1x128_e5m6(x.data_ptr(), m, k, ldx, q.data_ptr(), k * 3 // 2, s.data_ptr(), s.stride(0),
                                      s.stride(1), _stream())
    _check(st, "ds3_quant_act_1x128_e5m6")
    return q, s


def ds3_dequant_e5m6(q: torch.Tensor, s: torch.Tensor):
    """Packed E5M6 codes [M][3K/2] and scales -> BF16 [M][K]."""
    m, kb3, ldq = _rows2d(q, "q")
    k = kb3 * 2 // 3
    y = torch.empty((m, k), dtype=torch.bfloat16, device=q.device)
    st = _L().ds3_dequant_e5m6(q.data_ptr(), m, k, ldq, s.data_ptr(), s.stride(0), s.stride(1), y.data_ptr(), k, _stream())
    _check(st, "ds3_dequant_e5m6")
    return y


def ds3_adamw_bf16_states(master_w, grad, m, v, lr, beta1, beta2, eps, weight_decay, step, w_bf16=None):
    """One AdamW step in place: master_w FP32, grad FP32, m and v BF16 (all flat, same length, contiguous);
    w_bf16 (optional, BF16) receives the rounded new weights."""
    n = master_w.numel()
    ok = (master_w.dtype == torch.float32 and grad.dtype == torch.float32 and m.dtype == torch.bfloat16
          and v.dtype == torch.bfloat16 and grad.numel() == n and m.numel() == n and v.numel() == n)
    ok = ok and all(t.is_contiguous() for t in (master_w, grad, m, v))
    if w_bf16 is not None:
        ok = ok and w_bf16.dtype == torch.bfloat16 and w_bf16.numel() == n and w_bf16.is_contiguous()
    if not ok:
        raise TypeError("master_w, grad: FP32; m, v[, w_bf16]: BF16; all contiguous and of one length")
    st = _L().ds3_adamw_bf16_states(n, master_w.data_ptr(), grad.data_ptr(), m.data_ptr(), v.data_ptr(),
                                    w_bf16.data_ptr() if w_bf16 is not None else None, float(lr), float(beta1),
                                    float(beta2), float(eps), float(weight_decay), int(step), _stream())
    _check(st, "ds3_adamw_bf16_states")


def _swiglu_quant(entry: str, h: torch.Tensor, k_major_scales: bool):
    rows, two_i, ldh = _rows2d(h, "h")
    if h.dtype != torch.bfloat16 or two_i % 2:
        raise TypeError("h must be BF16 with an even number of columns")
    inter = two_i // 2
    q = _codes(rows, inter, h.device)
    s = _scales(rows, (inter + 127) // 128, h.device, k_major_scales)
    st = getattr(_L(), entry)(h.data_ptr(), rows, inter, ldh, q.data_ptr(), (inter + 15) // 16 * 16,
                              s.data_ptr(), s.stride(0), s.stride(1), _stream())
    _check(st, entry)
    return q, s


def ds3_swiglu_quant_1x128(h: torch.Tensor, k_major_scales: bool = True):
    """h [rows][2*inter] BF16 (gate | up) -> 1x128-quantized silu(gate) * up: (codes [rows][inter], scales)."""
    return _swiglu_quant("ds3_swiglu_quant_1x128", h, k_major_scales)


def ds3_swiglu_quant_1x128_pow2(h: torch.Tensor, k_major_scales: bool = True):
    """As ds3_swiglu_quant_1x128 with power-of-two scales."""
    return _swiglu_quant("ds3_swiglu_quant_1x128_pow2", h, k_major_scales)


def _grouped_swiglu_quant(entry, a, sa, group_offsets, b, sb, k_major_scales, workspace="auto"):
    m, k, lda = _rows2d(a, "a")
    g, n, kk = b.shape
    if kk != k or n % 256 or not b.is_contiguous() or not sb.is_contiguous():
        raise ValueError("b must be contiguous [G][2*inter][K] with inter % 128 == 0, sb contiguous")
    if group_offsets.dtype != torch.int32 or group_offsets.numel() != g + 1:
        raise ValueError("group_offsets must be int32 of length G+1")
    inter = n // 2
    q = _codes(m, inter, a.device)
    s = _scales(m, inter // 128, a.device, k_major_scales)
    st = getattr(_L(), entry)(g, group_offsets.data_ptr(), m, inter, k, a.data_ptr(), lda, sa.data_ptr(), sa.stride(0),
                              sa.stride(1), b.data_ptr(), k, sb.data_ptr(), q.data_ptr(), inter, s.data_ptr(),
                              s.stride(0), s.stride(1), *_grouped_ws(workspace, a.device), _stream())
    _check(st, entry)
    return q, s


def ds3_grouped_gemm_swiglu_quant_fp8_bs(a, sa, group_offsets, b, sb, k_major_scales: bool = True, workspace="auto"):
    """Grouped gate|up projection with SwiGLU and the 1x128 quantizer in its epilogue.
    b: [G][2*inter][K] codes with gate and up rows interleaved in blocks of 128
    (128 gate rows, the 128 up rows of the same range, ...), sb in the same order.
    Returns (codes [rows][inter], scales) of silu(gate) * up; rows beyond the last group are not written."""
    return _grouped_swiglu_quant("ds3_grouped_gemm_swiglu_quant_fp8_bs", a, sa, group_offsets, b, sb, k_major_scales, workspace)


def ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2(a, sa, group_offsets, b, sb, k_major_scales: bool = True, workspace="auto"):
    """As ds3_grouped_gemm_swiglu_quant_fp8_bs: power-of-two scales in, power-of-two scales out."""
    return _grouped_swiglu_quant("ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2", a, sa, group_offsets, b, sb, k_major_scales,
                                 workspace)


def _retile(entry: str, q: torch.Tensor, s: torch.Tensor, k_major_scales: bool):
    t, c, ldq = _rows2d(q, "q")
    if q.dtype != torch.uint8 or s.dtype != torch.float32 or tuple(s.shape) != (t, (c + 127) // 128):
        raise ValueError("q: uint8 [T][C]; s: float32 logical [T][ceil(C/128)]")
    q_t = _codes(c, t, q.device)
    s_t = _scales(c, (t + 127) // 128, q.device, k_major_scales)
    st = getattr(_L(), entry)(q.data_ptr(), t, c, ldq, s.data_ptr(), s.stride(0), s.stride(1), q_t.data_ptr(),
                              (t + 15) // 16 * 16, s_t.data_ptr(), s_t.stride(0), s_t.stride(1), _stream())
    _check(st, entry)
    return q_t, s_t


def ds3_retile_1x128_to_128x1(q: torch.Tensor, s: torch.Tensor, k_major_scales: bool = True):
    """1x128-quantized [T][C] (codes, scales) -> 128x1-quantized, transposed: (codes [C][T], scales [C][ceil(T/128)])."""
    return _retile("ds3_retile_1x128_to_128x1", q, s, k_major_scales)


def ds3_retile_1x128_to_128x1_pow2(q: torch.Tensor, s: torch.Tensor, k_major_scales: bool = True):
    """As ds3_retile_1x128_to_128x1 with power-of-two output scales."""
    return _retile("ds3_retile_1x128_to_128x1_pow2", q, s, k_major_scales)


def ds3_gemm_num_variants() -> int:
    return int(_L().ds3_gemm_num_variants())


def ds3_gemm_fp8_bs_noalloc(a, sa, b, sb, c: torch.Tensor, sb_mode: int = DS3_BSCALE_128x128, accumulate: bool = False):
    """ds3_gemm_fp8_bs into the caller's `c` through the entry point that allocates nothing."""
    m, k, lda = _rows2d(a, "a")
    n, kb_, ldb = _rows2d(b, "b")
    if kb_ != k or tuple(c.shape) != (m, n):
        raise ValueError("shapes disagree")
    _, _, ldc = _rows2d(c, "c")
    st = _L().ds3_gemm_fp8_bs_noalloc(m, n, k, a.data_ptr(), lda, sa.data_ptr(), sa.stride(0), sa.stride(1), b.data_ptr(), ldb,
                                      sb.data_ptr(), sb.stride(0), sb.stride(1), sb_mode, c.data_ptr(), _dt(c), ldc,
                                      int(accumulate), _stream())
    _check(st, "ds3_gemm_fp8_bs_noalloc")
    return c


def ds3_gemm_workspace_bytes(m: int, n: int, k: int) -> int:
    return int(_L().ds3_gemm_workspace_bytes(m, n, k))


def ds3_gemm_workspace_bytes_v(variant: int, m: int, n: int, k: int, sb_mode: int = DS3_BSCALE_128x128) -> int:
    return int(_L().ds3_gemm_workspace_bytes_v(variant, m, n, k, sb_mode))


def ds3_probe_mfma_fp8(iters: int, workgroups: int, out: torch.Tensor):
    """Enqueue the register-only FP8 MFMA loop (workgroups * 8 waves * iters * 32 MFMAs of 65536 flop)."""
    if out.dtype != torch.float32 or out.numel() < workgroups * 8:
        raise ValueError("out must hold workgroups * 8 floats")
    _check(_L().ds3_probe_mfma_fp8(iters, workgroups, out.data_ptr(), _stream()), "ds3_probe_mfma_fp8")


def ds3_probe_lds_feed(src: torch.Tensor, row_stride: int, iters: int, workgroups: int, out: torch.Tensor):
    """Enqueue the L2 -> LDS streaming loop (each workgroup moves iters * 64 KiB)."""
    if src.dtype != torch.uint8 or not src.is_contiguous() or out.dtype != torch.int32 or out.numel() < workgroups:
        raise ValueError("src: contiguous uint8; out: int32 of at least `workgroups` elements")
    _check(_L().ds3_probe_lds_feed(src.data_ptr(), src.numel(), row_stride, iters, workgroups, out.data_ptr(), _stream()),
           "ds3_probe_lds_feed")
