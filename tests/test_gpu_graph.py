"""The entry points enqueue work on the caller's stream and neither allocate nor
synchronise, so a sequence of them can be captured into a HIP graph.  The graph is
replayed several times with the program's own eager work and synchronisations in
between, and every replay is checked bit for bit against the eager result."""
import numpy as np
import pytest
import torch

from synth import workloads as wl
from tests._gpu_util import announce, dev

pytestmark = pytest.mark.gpu


def test_quantize_and_gemm_in_a_captured_graph(ds3):
    announce("graph capture")
    L = ds3._L()
    M, N, K = 384, 640, 1024
    x = dev(wl.cfg2_x(m=M, k=K), bf16=True)
    w = dev(wl.cfg2_w(n=N, k=K), bf16=True)
    qa = torch.empty((M, K), dtype=torch.uint8, device=x.device)
    sa = torch.empty((K // 128, M), dtype=torch.float32, device=x.device).t()
    qb = torch.empty((N, K), dtype=torch.uint8, device=x.device)
    sb = torch.empty((N // 128, K // 128), dtype=torch.float32, device=x.device)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    # this shape leaves a partial round of tiles, which the GEMM shares along K through the
    # workspace: the arrival counters are updated by every replay and left ready for the next
    ws_bytes = ds3.ds3_gemm_workspace_bytes(M, N, K)
    assert ws_bytes > 0
    ws = ds3.new_gemm_workspace(ws_bytes, x.device)     # prepared once, outside the graph

    def enqueue(stream):
        r = L.ds3_quant_act_1x128(x.data_ptr(), ds3.DS3_BF16, M, K, K, qa.data_ptr(), K, sa.data_ptr(), sa.stride(0), sa.stride(1), stream)
        r |= L.ds3_quant_w_128x128(w.data_ptr(), ds3.DS3_BF16, N, K, K, qb.data_ptr(), K, sb.data_ptr(), stream)
        r |= L.ds3_gemm_fp8_bs(M, N, K, qa.data_ptr(), K, sa.data_ptr(), sa.stride(0), sa.stride(1), qb.data_ptr(), K,
                               sb.data_ptr(), sb.stride(0), sb.stride(1), ds3.DS3_BSCALE_128x128, y.data_ptr(), ds3.DS3_BF16, N, 0,
                               ws.data_ptr(), ws_bytes, stream)
        assert r == 0

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(side.cuda_stream)                      # warm up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(torch.cuda.current_stream().cuda_stream)

    rng = np.random.default_rng(51)
    for it in range(4):
        # new inputs, eager reference on the default stream, some unrelated eager work, then the replay
        x.copy_(dev((wl.cfg2_x(m=M, k=K) * np.float32(rng.uniform(0.5, 2.0))).astype(np.float32), bf16=True))
        enqueue(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        want = (qa.clone(), sa.clone(), y.clone())
        qa.zero_(); y.zero_(); sa.zero_()
        _ = (x.float() @ x.float().t()).sum().item()   # eager work and a host synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(qa, want[0]) and torch.equal(sa, want[1]) and torch.equal(y, want[2]), it


def test_expert_ffn_in_a_captured_graph(ds3):
    """quantize -> grouped gate|up GEMM with SwiGLU and the cast in its epilogue -> grouped down GEMM,
    both GEMMs drawing their tiles from the queue in the workspace (one atomic per tile, counters put
    back by the last workgroup): every replay must equal the eager result bit for bit."""
    announce("graph capture: expert FFN")
    L = ds3._L()
    sizes, off, _ = wl.cfg3_routing(tokens=2048, local=8)
    rows, H, I, G = int(off[-1]), 1024, 256, 8
    x = dev(wl.cfg3_tokens(rows, k=H), bf16=True)
    w13 = dev(wl.interleave_gate_up(wl.cfg3_w13(g=G, inter=I, k=H)), bf16=True)
    w2 = dev(wl.cfg3_w2(g=G, inter=I, k=H), bf16=True)
    q13, s13 = ds3.ds3_quant_w_128x128(w13.view(G * 2 * I, H))
    q2, s2 = ds3.ds3_quant_w_128x128(w2.view(G * H, I))
    offd = dev(off)
    qx = torch.empty((rows, H), dtype=torch.uint8, device=x.device)
    sx = torch.empty((H // 128, rows), dtype=torch.float32, device=x.device).t()
    qh = torch.empty((rows, I), dtype=torch.uint8, device=x.device)
    sh = torch.empty((I // 128, rows), dtype=torch.float32, device=x.device).t()
    y = torch.empty((rows, H), dtype=torch.bfloat16, device=x.device)
    ws_bytes = L.ds3_grouped_gemm_workspace_bytes()
    ws = ds3.new_gemm_workspace(ws_bytes, x.device)     # prepared once, outside the graph

    def enqueue(stream):
        r = L.ds3_quant_act_1x128(x.data_ptr(), ds3.DS3_BF16, rows, H, H, qx.data_ptr(), H, sx.data_ptr(), sx.stride(0), sx.stride(1), stream)
        r |= L.ds3_grouped_gemm_swiglu_quant_fp8_bs(G, offd.data_ptr(), rows, I, H, qx.data_ptr(), H, sx.data_ptr(), sx.stride(0),
                                                    sx.stride(1), q13.data_ptr(), H, s13.data_ptr(), qh.data_ptr(), I, sh.data_ptr(),
                                                    sh.stride(0), sh.stride(1), ws.data_ptr(), ws_bytes, stream)
        r |= L.ds3_grouped_gemm_fp8_bs(G, offd.data_ptr(), rows, H, I, qh.data_ptr(), I, sh.data_ptr(), sh.stride(0), sh.stride(1),
                                       q2.data_ptr(), I, s2.data_ptr(), y.data_ptr(), ds3.DS3_BF16, H, ws.data_ptr(), ws_bytes, stream)
        assert r == 0

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(torch.cuda.current_stream().cuda_stream)
    rng = np.random.default_rng(52)
    for it in range(4):
        x.copy_(dev((wl.cfg3_tokens(rows, k=H) * np.float32(rng.uniform(0.5, 2.0))).astype(np.float32), bf16=True))
        enqueue(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        want = (qh.clone(), sh.clone(), y.clone())
        qh.zero_(); sh.zero_(); y.zero_()
        _ = (x.float() @ x.float().t()).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(qh, want[0]) and torch.equal(sh, want[1]) and torch.equal(y, want[2]), it
