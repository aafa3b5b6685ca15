"""The entry points under HIP graph capture: the library allocates nothing, synchronises nothing and clears memory with
kernels only, so a captured call must replay to exactly what the eager call gives -- on every replay, with new inputs in
the same buffers and eager work between the replays (the density dispatch included: its flag is written and read on the
device, inside the graph)."""
import numpy as np
import pytest
import torch

import paper_2004_04729_amd as dbp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _replay_matches_eager(call, inputs, outputs, fresh_inputs, after_replay=None):
    """call(stream) launches the entry point; inputs/outputs: lists of tensors it reads/writes in place."""
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        call(s.cuda_stream)                                     # eager first: one-time function attributes are set outside the capture
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        call(torch.cuda.current_stream().cuda_stream)
    for rnd, new in enumerate(fresh_inputs):
        for t, v in zip(inputs, new):
            t.copy_(v)
        for o in outputs:
            o.fill_(0)
        torch.cuda.synchronize()
        call(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        want = [o.clone() for o in outputs]
        for o in outputs:
            o.fill_(0)
        (torch.ones(1 << 20, device=DEV) * 2).sum().item()      # the program's own eager work between replays
        g.replay()
        torch.cuda.synchronize()
        for i, (o, w) in enumerate(zip(outputs, want)):
            assert torch.equal(o, w), "replay %d: output %d differs from the eager call" % (rnd, i)
        if after_replay:
            after_replay(rnd)


@pytest.mark.parametrize("B,n_in,n_out,scales", [(256, 1024, 2048, (8.0, 4.0, 16.0)),
                                                 (256, 4096, 16384, (8.0, 200.0, 8.0))])    # the second shape arms the density gate
def test_fc_backward_replays_like_the_eager_call(B, n_in, n_out, scales):
    g = torch.Generator(device=DEV)
    g.manual_seed(B + n_out)
    d = torch.empty((B, n_out), device=DEV)
    W = torch.randn((n_out, n_in), device=DEV, generator=g) * 0.03
    X = torch.relu(torch.randn((B, n_in), device=DEV, generator=g))
    codes = torch.empty((B, n_out), dtype=torch.int8, device=DEV)
    dX = torch.empty((B, n_in), device=DEV)
    dW = torch.empty((n_out, n_in), device=DEV)
    st = torch.zeros(32, dtype=torch.uint8, device=DEV)
    ws = torch.empty(dbp.linear_workspace_bytes(B, n_in, n_out), dtype=torch.uint8, device=DEV)
    step = 8e-3

    def call(stream):
        dbp.dithered_linear_backward(d, W, X, dbp.F32, B, n_in, n_out, step, 3, 0, codes, dX, dW, ws, st, dbp.PATH_AUTO, stream)

    # Laplace-like gradients of different spread against the fixed step: different densities (and, on the wide layer, both
    # sides of the device's dispatch threshold) in the same captured graph
    fresh = []
    for sc in scales:
        e = torch.empty((B, n_out), device=DEV).exponential_(1.0, generator=g)
        sign = torch.empty((B, n_out), device=DEV).uniform_(-1, 1, generator=g).sign_()
        fresh.append([e * sign * (step / sc)])
    d.copy_(fresh[0][0])
    flags = []
    off = dbp.format_layout(B, n_out)["scratch_offset"] + 16384 * 16          # where a gated call leaves its decision
    ws[off:off + 4] = 255
    _replay_matches_eager(call, [d], [codes, dX, dW, st], fresh,
                          after_replay=lambda rnd: flags.append(int(ws[off:off + 4].cpu().numpy().view(np.int32)[0])))
    if n_out == 16384:
        assert flags == [0, 1, 0], flags                        # matrix cores, gather kernels, matrix cores: decided inside the graph
    else:
        assert flags == [-1, -1, -1], flags                     # no gate on this shape: the word is never written


def test_conv_backward_and_static_quantiser_replay_like_the_eager_calls():
    N, C, H, Wd, K = 8, 64, 28, 28, 96
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    d = torch.empty((N, K, H, Wd), device=DEV)
    W = torch.randn((K, C, 3, 3), device=DEV, generator=g) * 0.05
    X = torch.relu(torch.randn((N, C, H, Wd), device=DEV, generator=g))
    codes = torch.empty((N, K, H, Wd), dtype=torch.int8, device=DEV)
    codes2 = torch.empty((N, K, H, Wd), dtype=torch.int8, device=DEV)
    dX = torch.empty_like(X)
    dW = torch.empty_like(W)
    st = torch.zeros(32, dtype=torch.uint8, device=DEV)
    st2 = torch.zeros(32, dtype=torch.uint8, device=DEV)
    ws = torch.empty(dbp.conv2d_workspace_bytes(N, C, H, Wd, K, 3, 3, 1, 1), dtype=torch.uint8, device=DEV)

    def call(stream):
        dbp.dithered_conv2d_backward(d, W, X, dbp.F32, N, C, H, Wd, K, 3, 3, 1, 1, 4e-3, 11, 0, codes, dX, dW, ws, st, dbp.PATH_AUTO, stream)
        dbp.nsd_quantize_static(d, N * K, H * Wd, 2e-3, 12, 0, codes2, st2, stream)

    fresh = [[torch.randn((N, K, H, Wd), device=DEV, generator=g) * sc] for sc in (1e-3, 3e-3, 5e-4)]
    d.copy_(fresh[0][0])
    _replay_matches_eager(call, [d], [codes, dX, dW, st, codes2, st2], fresh)


def test_conv_backward_with_the_dw_gate_replays_like_the_eager_call():
    # a layer that arms the middle state of the density gate (dX on matrix cores, dW on the plane-scanning gather kernel):
    # every candidate kernel is in the captured graph and the flags written inside it pick, replay by replay
    N, C, H, Wd, K = 64, 256, 14, 14, 256
    g = torch.Generator(device=DEV)
    g.manual_seed(9)
    d = torch.empty((N, K, H, Wd), device=DEV)
    W = torch.randn((K, C, 3, 3), device=DEV, generator=g) * 0.03
    X = torch.relu(torch.randn((N, C, H, Wd), device=DEV, generator=g))
    codes = torch.empty((N, K, H, Wd), dtype=torch.int8, device=DEV)
    dX = torch.empty_like(X)
    dW = torch.empty_like(W)
    st = torch.zeros(32, dtype=torch.uint8, device=DEV)
    ws = torch.empty(dbp.conv2d_workspace_bytes(N, C, H, Wd, K, 3, 3, 1, 1), dtype=torch.uint8, device=DEV)

    def call(stream):
        dbp.dithered_conv2d_backward(d, W, X, dbp.F32, N, C, H, Wd, K, 3, 3, 1, 1, 4e-3, 11, 0, codes, dX, dW, ws, st, dbp.PATH_AUTO, stream)

    fresh = [[torch.randn((N, K, H, Wd), device=DEV, generator=g) * sc] for sc in (1e-3, 5e-5, 4e-4)]    # ~20 %, ~1 %, ~8 % nonzeros
    d.copy_(fresh[0][0])
    flags = []
    off = dbp.format_layout(N * K, H * Wd)["scratch_offset"] + 16384 * 16
    ws[off:off + 12] = 255
    _replay_matches_eager(call, [d], [codes, dX, dW, st], fresh,
                          after_replay=lambda rnd: flags.append([int(v) for v in ws[off:off + 12].cpu().numpy().view(np.int32)]))
    assert flags == [[0, 0, 1], [0, 1, 0], [0, 0, 1]], flags
