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
