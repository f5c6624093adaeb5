"""The library under HIP graph capture: it allocates nothing and launches only kernels, so a
forward + backward pair can be captured once and replayed; every replay must equal the eager result."""
import numpy as np
import pytest

from paper_2501_06480_amd import synth
from gpu_util import f32_device, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("L,heads,d,N,dbias", [(49, 12, 32, 512, True), (144, 4, 32, 64, False), (64, 4, 64, 128, True)])
def test_captured_forward_backward_replays_match_eager(L, heads, d, N, dbias):
    import torch
    import paper_2501_06480_amd as fwa
    w = synth.Workload(f"graph_L{L}", N, L, heads * d, heads, "bf16", 9300 + L, 0, backward=True)
    bias = f32_device(synth.normal((heads, L, L), 73 + L, 0.5))
    m = np.where(synth.rng(79 + L).random((4, L, L)) < 0.2, -100.0, 0.0).astype(np.float32)
    m[:, np.arange(L), np.arange(L)] = 0.0
    mask = f32_device(m)
    shape = (N, L, heads * d)
    q, k, v, g = (torch.zeros(shape, dtype=torch.bfloat16, device="cuda") for _ in range(4))
    o, dq, dk, dv = (torch.empty(shape, dtype=torch.bfloat16, device="cuda") for _ in range(4))
    need = fwa.fwa_backward_workspace_bytes(N, L, heads * d, heads, 1, dbias)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def run(stream=None):
        fwa.fwa_forward(q, k, v, heads, w.scale, bias, mask, out=o, stream=stream)
        return fwa.fwa_backward(q, k, v, g, heads, w.scale, bias, mask, want_dbias=dbias, workspace=ws,
                                out=(dq, dk, dv), stream=stream)[3]

    def fill(seed):
        x = synth.draw(synth.Workload(w.name, N, L, heads * d, heads, "bf16", seed, 0, backward=True))
        for t, nme in ((q, "q"), (k, "k"), (v, "v"), (g, "d_o")):
            t.copy_(to_device(x, w, nme))

    fill(1)
    run()                     # warm-up outside the capture (first-call attribute queries)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    # dBias is allocated by the binding per call; inside the capture it comes from the graph's pool
    with torch.cuda.graph(graph, stream=side):
        db_graph = run(torch.cuda.current_stream())
    for seed in (2, 3, 4):
        fill(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (o, dq, dk, dv)] + ([db_graph.clone()] if dbias else [])
        for t in (o, dq, dk, dv):
            t.fill_(7.0)
        db_eager = run()
        torch.cuda.synchronize()
        want = [o, dq, dk, dv] + ([db_eager] if dbias else [])
        for a, b in zip(got, want):
            assert torch.equal(a, b), seed


@pytest.mark.parametrize("L,heads,N,nW,bf16_bias", [(144, 4, 64, 16, True),      # the bias widened into the workspace
                                                    (49, 3, 1024, 512, False),   # per-window masks from the labels
                                                    (49, 6, 1024, 512, True)])
def test_captured_label_calls_replay(L, heads, N, nW, bf16_bias):
    """The label entry points under capture: the fp32 copy of a bf16 bias (a kernel writing into the
    workspace) and the per-window label fetches are part of the graph like everything else."""
    import torch
    import paper_2501_06480_amd as fwa
    C = 32 * heads
    w = synth.Workload(f"graph_labels_L{L}", N, L, C, heads, "bf16", 9400 + L + heads, 0, backward=True)
    bias = f32_device(synth.normal((heads, L, L), 83 + L, 0.5))
    if bf16_bias:
        bias = bias.bfloat16()
    labels = torch.from_numpy(synth.rng(89 + L).integers(0, 4, (nW, L)).astype(np.int32)).cuda()
    shape = (N, L, C)
    q, k, v, g = (torch.zeros(shape, dtype=torch.bfloat16, device="cuda") for _ in range(4))
    o, dq, dk, dv = (torch.empty(shape, dtype=torch.bfloat16, device="cuda") for _ in range(4))
    ws = torch.empty(fwa.fwa_backward_workspace_bytes(N, L, C, heads, 1, True), dtype=torch.uint8, device="cuda")

    def run(stream=None):
        fwa.fwa_forward(q, k, v, heads, w.scale, bias, labels=labels, out=o, stream=stream)
        return fwa.fwa_backward(q, k, v, g, heads, w.scale, bias, labels=labels, want_dbias=True, workspace=ws,
                                out=(dq, dk, dv), stream=stream)[3]

    def fill(seed):
        x = synth.draw(synth.Workload(w.name, N, L, C, heads, "bf16", seed, 0, backward=True))
        for t, nme in ((q, "q"), (k, "k"), (v, "v"), (g, "d_o")):
            t.copy_(to_device(x, w, nme))

    fill(1)
    run()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        db_graph = run(torch.cuda.current_stream())
    for seed in (2, 3, 4):
        fill(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (o, dq, dk, dv, db_graph)]
        for t in (o, dq, dk, dv):
            t.fill_(7.0)
        ws.fill_(0x5a)   # the workspace carries nothing from one call to the next
        db_eager = run()
        torch.cuda.synchronize()
        for a, b in zip(got, [o, dq, dk, dv, db_eager]):
            assert torch.equal(a, b), seed
