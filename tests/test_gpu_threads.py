"""Calls from several host threads on streams of their own: the library keeps no state between calls
(options and the per-thread diagnostics aside), so concurrent callers must each get the oracle's bits."""
import threading

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


def test_concurrent_callers_on_their_own_streams(mad):
    import torch
    # different shapes: different kernels of the library in flight at once
    shapes = [(20000, 512, 256, 32), (5000, 64, 24, 8), (17000, 510, 250, 30), (3000, 128, 100, 32)]
    jobs = []
    for k, (N, D, M, C) in enumerate(shapes):
        rng = np.random.default_rng(100 + k)
        _, A, B = wl.random_problem(N + k, N, D, M, latent=8, N_train=4)
        sd, th = random_trees(rng, A, C)
        P = rng.standard_normal((C, 16, D)).astype(np.float32)
        luts, scale, offset, _, _ = oracle.quantize_luts(oracle.build_luts_f64(P, B))
        want_out, want_acc, want_packed = oracle.encode_scan(A, sd, th, luts, scale, offset)
        jobs.append(dict(shape=(N, D, M, C), A=A, sd=sd, th=th, P=P, luts=luts, scale=scale, offset=offset,
                         want_out=want_out, want_packed=want_packed))
    errors = []
    barrier = threading.Barrier(len(jobs))

    def worker(job):
        try:
            dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                params = mad.Params(dev(job["sd"]), dev(job["th"]), dev(job["P"]))
                A_d, luts, scale, offset = dev(job["A"]), dev(job["luts"]), dev(job["scale"]), dev(job["offset"])
                stream.synchronize()
                barrier.wait(timeout=60)
                for rep in range(20):
                    codes = mad.maddness_encode(params, A_d)
                    out_f = mad.maddness_encode_scan(params, A_d, luts, scale, offset)
                    out_s, _ = mad.maddness_scan(job["shape"][3], codes, luts, scale, offset)
                    stream.synchronize()
                    if not (codes.cpu().numpy() == job["want_packed"]).all():
                        errors.append((job["shape"], rep, "codes"))
                    if not (out_f.cpu().numpy() == job["want_out"]).all():
                        errors.append((job["shape"], rep, "fused out"))
                    if not (out_s.cpu().numpy() == job["want_out"]).all():
                        errors.append((job["shape"], rep, "scan out"))
        except Exception as e:   # a failed call in a thread must fail the test
            errors.append((job["shape"], repr(e)))

    threads = [threading.Thread(target=worker, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=300)
    assert not any(t.is_alive() for t in threads), "a caller did not finish"
    assert not errors, errors[:5]
