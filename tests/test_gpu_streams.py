"""The library only enqueues kernels on the stream it is given: it must work on a non-default stream and
inside a captured HIP graph (it allocates nothing, synchronises nothing and issues no memset)."""
import numpy as np
import pytest
import torch

import synth_inputs as synth
from _util import to_gpu_bf16

pytestmark = pytest.mark.gpu


def _step(uly, t, scale):
    o, lse = uly.ulysses_attn_fwd(t[0], t[1], t[2], scale, True)
    return (o, lse) + tuple(uly.ulysses_attn_bwd(t[0], t[1], t[2], o, t[3], lse, scale, True))


def test_side_stream_gives_the_same_bits(gpu_lib):
    q, k, v, do = synth.attention_inputs(700, 2, 128, 3)
    t = [to_gpu_bf16(a) for a in (q, k, v, do)]
    ref = _step(gpu_lib, t, 0.09)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        got = _step(gpu_lib, t, 0.09)
    side.synchronize()
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


def test_graph_capture_and_replay(gpu_lib):
    N, Hl, d, scale = 600, 2, 64, 0.125
    q, k, v, do = synth.attention_inputs(N, Hl, d, 4)
    t = [to_gpu_bf16(a) for a in (q, k, v, do)]
    o = torch.empty_like(t[0]); lse = torch.empty((Hl, N), dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(t[0]) for _ in range(3))
    ws = torch.empty(gpu_lib.ulysses_attn_bwd_workspace_bytes(N, Hl, d), dtype=torch.uint8, device="cuda")

    def run():
        gpu_lib.ulysses_attn_fwd(t[0], t[1], t[2], scale, True, out=o, lse=lse)
        gpu_lib.ulysses_attn_bwd(t[0], t[1], t[2], o, t[3], lse, scale, True, workspace=ws, out=grads)

    run()
    torch.cuda.synchronize()
    ref = [x.clone() for x in (o, lse) + grads]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    for rep in range(4):
        for x in (o, lse) + grads:
            x.zero_()                                   # eager work between the replays
        t[0].add_(0)                                     # (and a harmless eager kernel on the inputs)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, (o, lse) + grads):
            assert torch.equal(a, b), rep


def _window_global(nb, w):
    i, j = np.indices((nb, nb))
    return np.tril((i - j < w) | (j == 0))


def test_sparse_backward_workspace_is_rebuilt_by_every_call(gpu_lib):
    """The sparse backward keeps its work plan and partial sums in the caller's workspace: a call must not
    depend on what an earlier call with another pattern left there."""
    N, Hl, d, scale = 5000, 2, 128, 0.09
    nb = (N + gpu_lib.SPARSE_BLOCK - 1) // gpu_lib.SPARSE_BLOCK
    t = [to_gpu_bf16(a) for a in synth.attention_inputs(N, Hl, d, 6)]
    ws = torch.empty(gpu_lib.ulysses_sparse_attn_bwd_workspace_bytes(N, Hl, d), dtype=torch.uint8, device="cuda")
    pats = [gpu_lib.SparsePattern(m) for m in (_window_global(nb, 2), np.ones((nb, nb), bool), np.eye(nb, dtype=bool))]
    for pat in pats + pats[::-1]:
        o, lse = gpu_lib.ulysses_sparse_attn_fwd(t[0], t[1], t[2], pat, scale)
        fresh = gpu_lib.ulysses_sparse_attn_bwd(t[0], t[1], t[2], o, t[3], lse, pat, scale)
        reused = gpu_lib.ulysses_sparse_attn_bwd(t[0], t[1], t[2], o, t[3], lse, pat, scale, workspace=ws)
        for a, b in zip(fresh, reused):
            assert torch.equal(a, b)


def test_sparse_graph_capture_and_replay(gpu_lib):
    """Plan, work items and the reduction of cut block columns are plain launches: they replay from a graph."""
    N, Hl, d, scale = 5000, 2, 128, 0.09
    nb = (N + gpu_lib.SPARSE_BLOCK - 1) // gpu_lib.SPARSE_BLOCK
    pat = gpu_lib.SparsePattern(_window_global(nb, 3))
    t = [to_gpu_bf16(a) for a in synth.attention_inputs(N, Hl, d, 7)]
    o = torch.empty_like(t[0]); lse = torch.empty((Hl, N), dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(t[0]) for _ in range(3))
    ws = torch.empty(gpu_lib.ulysses_sparse_attn_bwd_workspace_bytes(N, Hl, d), dtype=torch.uint8, device="cuda")
    fws = torch.empty(gpu_lib.ulysses_sparse_attn_fwd_workspace_bytes(N, Hl, d), dtype=torch.uint8, device="cuda")

    def run():
        gpu_lib.ulysses_sparse_attn_fwd(t[0], t[1], t[2], pat, scale, out=o, lse=lse, workspace=fws)
        gpu_lib.ulysses_sparse_attn_bwd(t[0], t[1], t[2], o, t[3], lse, pat, scale, workspace=ws, out=grads)

    run()
    torch.cuda.synchronize()
    ref = [x.clone() for x in (o, lse) + grads]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    for rep in range(3):
        for x in (o, lse) + grads:
            x.zero_()
        ws.fill_(rep + 1)                                # whatever the workspaces hold, the replay rebuilds it
        fws.fill_(rep + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, (o, lse) + grads):
            assert torch.equal(a, b), rep
