"""Nothing is written outside what a call owns: padding columns of the code arrays (leading
dimension beyond the row), the row past the last one, and the floats around the scale arrays
keep their sentinel values.  Raw C ABI with explicit leading dimensions."""
import numpy as np
import pytest
import torch

from tests._gpu_util import announce, dev

pytestmark = pytest.mark.gpu

SENT = 0xCD
FSENT = -12345.5


def _codes(rows, ld):
    return torch.full((rows + 1, ld), SENT, dtype=torch.uint8, device="cuda:0")      # one spare row


def _check_codes(buf, rows, cols, what):
    h = buf.cpu().numpy()
    assert np.all(h[:rows, cols:] == SENT), f"{what}: padding columns written"
    assert np.all(h[rows:] == SENT), f"{what}: row past the end written"
    assert not np.all(h[:rows, :cols] == SENT), f"{what}: nothing written"


def _scales(n):
    return torch.full((n + 64,), FSENT, dtype=torch.float32, device="cuda:0")        # 32 floats of guard on either side


def _check_scales(buf, n, what):
    h = buf.cpu().numpy()
    assert np.all(h[:32] == FSENT) and np.all(h[32 + n:] == FSENT), f"{what}: scale guard written"
    assert not np.any(h[32:32 + n] == FSENT), f"{what}: a scale was not written"


@pytest.mark.parametrize("rows,cols", [(130, 1160), (16, 128), (37, 136)])
def test_quantizers_stay_inside_their_outputs(ds3, rows, cols):
    announce(f"guard bands {rows}x{cols}")
    L = ds3._L()
    st = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(81)
    x = dev(rng.standard_normal((rows, cols)).astype(np.float32), bf16=True)
    nkb, ntb, nrb = (cols + 127) // 128, (rows + 127) // 128, (rows + 127) // 128
    ldq = (cols + 15) // 16 * 16 + 32
    for entry in ("ds3_quant_act_1x128", "ds3_quant_act_1x128_pow2"):
        for k_major in (True, False):
            q, s = _codes(rows, ldq), _scales(rows * nkb)
            sr, sk = (1, rows) if k_major else (nkb, 1)
            assert getattr(L, entry)(x.data_ptr(), ds3.DS3_BF16, rows, cols, cols, q.data_ptr(), ldq, s.data_ptr() + 128, sr, sk, st) == 0
            _check_codes(q, rows, cols, entry)
            _check_scales(s, rows * nkb, entry)
    # 128x128 and its dual-layout form
    q, s = _codes(rows, ldq), _scales(nrb * nkb)
    assert L.ds3_quant_w_128x128(x.data_ptr(), ds3.DS3_BF16, rows, cols, cols, q.data_ptr(), ldq, s.data_ptr() + 128, st) == 0
    _check_codes(q, rows, cols, "128x128")
    _check_scales(s, nrb * nkb, "128x128")
    ldt = (rows + 15) // 16 * 16 + 16
    q, s, qt, s_t = _codes(rows, ldq), _scales(nrb * nkb), _codes(cols, ldt), _scales(nrb * nkb)
    assert L.ds3_quant_w_128x128_dual(x.data_ptr(), ds3.DS3_BF16, rows, cols, cols, q.data_ptr(), ldq, s.data_ptr() + 128,
                                      qt.data_ptr(), ldt, s_t.data_ptr() + 128, st) == 0
    _check_codes(q, rows, cols, "dual"); _check_codes(qt, cols, rows, "dual transposed")
    _check_scales(s, nrb * nkb, "dual"); _check_scales(s_t, nrb * nkb, "dual transposed")
    # 128x1: codes [cols][ld >= rows], scales [cols][ntb]
    qt, s_t = _codes(cols, ldt), _scales(cols * ntb)
    assert L.ds3_quant_act_128x1(x.data_ptr(), ds3.DS3_BF16, rows, cols, cols, qt.data_ptr(), ldt, s_t.data_ptr() + 128, 1, cols, st) == 0
    _check_codes(qt, cols, rows, "128x1")
    _check_scales(s_t, cols * ntb, "128x1")
    # cache re-tiling: 1x128 codes and scales in, 128x1 out
    q1, s1 = ds3.ds3_quant_act_1x128(x)
    if cols % 16 == 0:
        qt, s_t = _codes(cols, ldt), _scales(cols * ntb)
        assert L.ds3_retile_1x128_to_128x1(q1.data_ptr(), rows, cols, q1.stride(0), s1.data_ptr(), s1.stride(0), s1.stride(1),
                                           qt.data_ptr(), ldt, s_t.data_ptr() + 128, 1, cols, st) == 0
        _check_codes(qt, cols, rows, "retile")
        _check_scales(s_t, cols * ntb, "retile")
    # fused producers
    if cols % 16 == 0:
        inter = cols // 2
        nib = (inter + 127) // 128
        ldi = (inter + 15) // 16 * 16 + 16
        q, s = _codes(rows, ldi), _scales(rows * nib)
        assert L.ds3_swiglu_quant_1x128(x.data_ptr(), rows, inter, cols, q.data_ptr(), ldi, s.data_ptr() + 128, 1, rows, st) == 0
        _check_codes(q, rows, inter, "swiglu->quant")
        _check_scales(s, rows * nib, "swiglu->quant")
    gamma = torch.ones(cols, dtype=torch.float32, device="cuda:0")
    q, s = _codes(rows, ldq), _scales(rows * nkb)
    y = torch.full((rows + 1, cols + 8), 7.0, dtype=torch.bfloat16, device="cuda:0")
    assert L.ds3_rmsnorm_quant_1x128(x.data_ptr(), rows, cols, cols, gamma.data_ptr(), 1e-6, y.data_ptr(), cols + 8, q.data_ptr(), ldq,
                                     s.data_ptr() + 128, 1, rows, st) == 0
    _check_codes(q, rows, cols, "rmsnorm->quant")
    _check_scales(s, rows * nkb, "rmsnorm->quant")
    yh = y.float().cpu().numpy()
    assert np.all(yh[:rows, cols:] == 7.0) and np.all(yh[rows:] == 7.0)
    # E5M6 cache: 12-bit codes, 3 bytes per 2 elements
    ld6 = cols * 3 // 2 + 8
    q, s = _codes(rows, ld6), _scales(rows * nkb)
    assert L.ds3_quant_act_1x128_e5m6(x.data_ptr(), rows, cols, cols, q.data_ptr(), ld6, s.data_ptr() + 128, 1, rows, st) == 0
    _check_codes(q, rows, cols * 3 // 2, "e5m6")
    _check_scales(s, rows * nkb, "e5m6")
