"""The library's calls under HIP graph capture: they allocate nothing, read no host state at
replay and enqueue only kernels, so a captured table build + fused call must replay to the
bits of the eager calls, every time, also after the inputs have changed in place."""
import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import random_trees

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mad():
    import torch
    import paper_2106_10860_amd as m
    assert torch.cuda.is_available()
    m.lib()
    return m


@pytest.mark.parametrize("shape", [(3000, 64, 24, 8), (20000, 512, 256, 32), (10000, 512, 10, 16)],
                         ids=lambda s: "N%d_D%d_M%d_C%d" % s)
def test_captured_calls_replay_to_the_eager_bits(mad, shape):
    import torch
    N, D, M, C = shape
    rng = np.random.default_rng(N + M)
    _, A, B = wl.random_problem(N + 17, N, D, M, latent=8, N_train=4)
    sd, th = random_trees(rng, A, C)
    P = rng.standard_normal((C, 16, D)).astype(np.float32)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    params = mad.Params(dev(sd), dev(th), dev(P))
    A_d, B_d = dev(A), dev(B)
    luts = torch.zeros((C, 16, M), dtype=torch.uint8, device="cuda")
    scale = torch.zeros(M, device="cuda")
    offset = torch.zeros(M, device="cuda")
    out = torch.zeros((N, M), device="cuda")
    codes = torch.zeros((N, C // 2), dtype=torch.uint8, device="cuda")

    def calls():
        mad.maddness_build_luts_static(params, B_d, luts, scale, offset)      # the workspace is the library's own
        mad.maddness_encode_scan(params, A_d, luts, scale, offset, out=out, codes=codes)

    calls()                      # eager: one-time kernel attributes are set here, outside the capture
    torch.cuda.synchronize()
    want_out, want_codes, want_luts = out.clone(), codes.clone(), luts.clone()
    T = oracle.build_luts_f64(P, B)
    luts_o, scale_o, offset_o, _, _ = oracle.quantize_luts(T)
    assert np.abs(want_luts.cpu().numpy().astype(int) - luts_o.astype(int)).max() <= 1

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            calls()
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(4):
        out.fill_(-1.0); codes.zero_(); luts.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want_out) and torch.equal(codes, want_codes) and torch.equal(luts, want_luts), replay
        # eager work of the program between the replays
        mad.maddness_encode(params, A_d)
        torch.cuda.synchronize()
    # new inputs in the same buffers: the replay computes on what the buffers hold now
    _, A2, B2 = wl.random_problem(N + 18, N, D, M, latent=8, N_train=4)
    A_d.copy_(dev(A2)); B_d.copy_(dev(B2))
    graph.replay()
    torch.cuda.synchronize()
    got_out, got_codes = out.clone(), codes.clone()
    calls()
    torch.cuda.synchronize()
    assert torch.equal(out, got_out) and torch.equal(codes, got_codes)
    want, _, packed = oracle.encode_scan(A2, sd, th, luts.cpu().numpy(), scale.cpu().numpy(), offset.cpu().numpy())
    assert (got_codes.cpu().numpy() == packed).all() and (got_out.cpu().numpy() == want).all()
