"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation), so a layer call
can be captured into a HIP graph and replayed.  The graph is replayed several times with the program's own
eager work and synchronisations between the replays, on changing inputs, and every replay is compared with the
eager result of the same input."""
import numpy as np
import pytest
import torch

import paper_2512_05409_amd as sq
import workloads
from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,mode,noalloc", [(8, "dynamic", False), (200, "dynamic", False), (48, "static", False),
                                             (300, "tied", False), (24, "dynamic", True), (150, "static", True)])
def test_sq_linear_under_graph_capture(M, mode, noalloc):
    """noalloc: the captured call is sq_linear_noalloc (its workspace is the library's fixed device array: the
    form of the layer for code that may not allocate, such as a capture)."""
    K, N, bank, topk = 1024, 384, 64, 8
    rng = np.random.Generator(np.random.PCG64([M, 99]))
    xs = [workloads.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32) * (1 + 20 * (rng.random((1, K)) < 0.02)))
          for _ in range(4)]
    wq = workloads.pack_int4(rng.integers(-8, 8, size=(N, K), dtype=np.int8))
    sw = rng.uniform(0.005, 0.02, size=N).astype(np.float32)
    static = mode == "static"
    lib_mode = {"dynamic": sq.SQ_DYNAMIC, "static": sq.SQ_STATIC, "tied": sq.SQ_DYNAMIC_TIED}[mode]
    p = sq.params(M, K, N, bank, topk, mode=lib_mode, out_dtype=sq.SQ_OUT_F32)
    wqd, swd = dev(wq), dev(sw)
    md, pre = None, None
    if static:
        mask = np.zeros(K // 32, np.uint32)
        for g in range(K // bank):
            for i in rng.choice(bank, topk, replace=False):
                j = g * bank + int(i)
                mask[j // 32] |= np.uint32(1 << (j % 32))
        md = dev(mask)
        pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
        sq.sq_weight_prepack(p, wqd, mask, md, pre)
    w = sq.weight(wqd, swd, pre)
    ws = torch.empty(sq.sq_linear_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    x_static = dev(xs[0]).clone()
    y_graph = torch.zeros(M * N, dtype=torch.float32, device="cuda")
    y_eager = torch.zeros(M * N, dtype=torch.float32, device="cuda")

    # eager references (also the first use of every kernel on this device, outside the capture)
    want = []
    for x in xs:
        x_static.copy_(dev(x))
        sq.sq_linear(p, x_static, w, y_eager, ws, static_mask=md)
        torch.cuda.synchronize()
        want.append(y_eager.cpu().numpy().copy())

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        x_static.copy_(dev(xs[0]))
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            if noalloc:
                sq.sq_linear_noalloc(p, x_static, w, y_graph, static_mask=md, stream=side)
            else:
                sq.sq_linear(p, x_static, w, y_graph, ws, static_mask=md, stream=side)
    torch.cuda.synchronize()

    for rep in range(2):
        for i, x in enumerate(xs):
            x_static.copy_(dev(x))
            y_graph.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = y_graph.cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want[i].view(np.uint32)), f"replay {rep}.{i}"
            # eager work between replays, on the same buffers
            sq.sq_linear(p, x_static, w, y_eager, ws, static_mask=md)
            torch.cuda.synchronize()
            assert np.array_equal(y_eager.cpu().numpy().view(np.uint32), want[i].view(np.uint32))
